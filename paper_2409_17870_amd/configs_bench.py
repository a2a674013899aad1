#!/usr/bin/env python3
"""Times every workload configuration of the problem statement and prices each against its roofline.

Run on an MI355X: ``python -m paper_2409_17870_amd.configs_bench [--configs 1,2,3,4,5]``.  Prints markdown.

Step of a configuration (what is inside the timed region):
  1, 2   GEMM with int32 output, and activation packing + GEMM
  3      decode shapes: GEMM straight from the activation codes (the online packing is part of the call), fp16
         output through the scale epilogue; weights pre-packed
  4      GEMM with int32 and fp16 outputs (activations pre-packed), and with the packing
  5      activation packing + GEMM with the fp16 epilogue, per linear and for the whole decoder-layer sweep

Two clocks per step: "calls" is a HIP event pair around a loop of back-to-back calls through the C ABI (the host's
launch cost is inside; for steps of a few microseconds that is all one sees), "graph" is the same loop captured once
into a HIP graph and replayed (what a serving loop that captures its decode step pays).  For the HBM-bound decode shapes
the loop walks over enough distinct packed weight copies (640 MiB) that neither L2 nor the memory-side cache serves them.

Roofline: t_roof = max(2 M N K / 5.0 POP/s, algorithmic bytes / 8 TB/s); bytes = packed weights + packed activations
+ outputs (+ the unpacked codes read and the packed activations written when packing is inside the step).
Integer GEMM time does not depend on the values, so codes are random; parity on these shapes is the tests' job.
"""
import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK = 5.0e15
HBM_PEAK = 8.0e12


def main():
    import torch
    from paper_2409_17870_amd import binding, inputs

    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    binding.load()

    def settle(step, ms=40.0):
        # after idling (data generation between cases) the GPU needs some tens of ms of work before its clocks settle
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < ms:
            for i in range(20):
                step(i)
            torch.cuda.synchronize()

    def clock_calls(step, iters):
        settle(step)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / iters

    def clock_graph(step, reps, replays=10):
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            step(0)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                for i in range(reps):
                    step(i)
            g.replay()
            torch.cuda.synchronize()
            settle(lambda i: g.replay() if i % 20 == 0 else None, ms=20.0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(replays):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (replays * reps)

    def row(label, case, us_calls, us_graph, nbytes):
        M, N, K = case["M"], case["N"], case["K"]
        ops = 2.0 * M * N * K
        t_roof = max(ops / INT8_PEAK, nbytes / HBM_PEAK) * 1e6
        bound = "int8 MFMA" if ops / INT8_PEAK > nbytes / HBM_PEAK else "HBM"
        best = min(us_calls, us_graph)
        print("| %s | %d | %d | %d | W%dA%d | %.1f | %.1f | %.0f | %.0f | %.2f (%s) | %.0f %% |" % (
            label, M, N, K, case["q"], case["p"], us_calls, us_graph, ops / best / 1e6, nbytes / best / 1e3,
            t_roof, bound, 100.0 * t_roof / best), flush=True)

    def operands(case, copies=1):
        M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        wp0 = binding.apmm_pack_weights(w, q)
        wps = [wp0] + [wp0.clone() for _ in range(copies - 1)]
        a_packed = binding.apmm_pack_activations(a, p)
        sa = (torch.rand(M, device=dev) * 0.09 + 0.01).half()
        sw = (torch.rand(N, device=dev) * 0.09 + 0.01).half()
        return a, a_packed, wps, sa, sw

    print("| step | M | N | K | scheme | calls (us) | graph (us) | eff. TOPS | GB/s | t_roof us (bound) | of roofline |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for idx in [int(x) for x in args.configs.split(",")]:
        sweep_calls = sweep_graph = 0.0
        for case in inputs.config_cases(idx):
            M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
            w_bytes, a_bytes = N * K * q / 8.0, M * K * p / 8.0
            pack_bytes = M * K + a_bytes
            iters = 200 if idx != 3 else 400
            if idx in (1, 2):
                a, a_packed, wps, sa, sw = operands(case)
                c = torch.empty((M, N), dtype=torch.int32, device=dev)

                def gemm(i):
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[0], c_i32=c)

                def pack_gemm(i):
                    binding.apmm_pack_activations(a, p, out=a_packed)
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[0], c_i32=c)

                nb = w_bytes + a_bytes + 4.0 * M * N
                row("cfg%d GEMM, int32" % idx, case, clock_calls(gemm, iters), clock_graph(gemm, 20), nb)
                row("cfg%d pack + GEMM, int32" % idx, case, clock_calls(pack_gemm, iters), clock_graph(pack_gemm, 20),
                    nb + pack_bytes)
            elif idx == 3:
                copies = max(2, int((640 << 20) // w_bytes))
                a, a_packed, wps, sa, sw = operands(case, copies)
                h = torch.empty((M, N), dtype=torch.float16, device=dev)

                def from_codes(i):
                    binding.apmm_gemm_from_codes(a, N, p, q, wps[i % copies], want_i32=False, want_f16=True,
                                                 w_scale=sw, a_scale=sa, c_f16=h, workspace=a_packed)

                def pack_gemm(i):
                    binding.apmm_pack_activations(a, p, out=a_packed)
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[i % copies], want_i32=False, want_f16=True,
                                      w_scale=sw, a_scale=sa, c_f16=h)

                nb = w_bytes + M * K + 2.0 * M * N + 2.0 * (M + N)
                row("cfg3 GEMM from codes, fp16", case, clock_calls(from_codes, iters), clock_graph(from_codes, copies), nb)
                row("cfg3 pack + GEMM, fp16", case, clock_calls(pack_gemm, iters), clock_graph(pack_gemm, copies),
                    nb + 2 * a_bytes)
            elif idx == 4:
                a, a_packed, wps, sa, sw = operands(case)
                c = torch.empty((M, N), dtype=torch.int32, device=dev)
                h = torch.empty((M, N), dtype=torch.float16, device=dev)

                def gemm(i):
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[0], want_f16=True, w_scale=sw, a_scale=sa,
                                      c_i32=c, c_f16=h)

                def pack_gemm(i):
                    binding.apmm_pack_activations(a, p, out=a_packed)
                    gemm(i)

                nb = w_bytes + a_bytes + 6.0 * M * N + 2.0 * (M + N)
                row("cfg4 GEMM, int32 + fp16", case, clock_calls(gemm, iters), clock_graph(gemm, 10), nb)
                row("cfg4 pack + GEMM, int32 + fp16", case, clock_calls(pack_gemm, iters), clock_graph(pack_gemm, 10),
                    nb + pack_bytes)
            else:
                a, a_packed, wps, sa, sw = operands(case)
                h = torch.empty((M, N), dtype=torch.float16, device=dev)

                def pack_gemm(i):
                    binding.apmm_pack_activations(a, p, out=a_packed)
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[0], want_i32=False, want_f16=True, w_scale=sw,
                                      a_scale=sa, c_f16=h)

                nb = w_bytes + a_bytes + 2.0 * M * N + 2.0 * (M + N) + pack_bytes
                tc, tg = clock_calls(pack_gemm, iters), clock_graph(pack_gemm, 10)
                sweep_calls += tc
                sweep_graph += tg
                row("cfg5 pack + GEMM, fp16", case, tc, tg, nb)
            del a, a_packed, wps
            torch.cuda.empty_cache()
        if idx == 5:
            # the same layer with the projections that share an input fused by concatenating their weights (what a
            # model would do: q,k,v -> one 15360-channel linear, gate,up -> one 27648-channel linear): four GEMMs
            fused_calls = fused_graph = 0.0
            for (name, N, K) in (("q,k,v fused", 15360, 5120), ("o", 5120, 5120), ("gate,up fused", 27648, 5120),
                                 ("down", 5120, 13824)):
                case = dict(M=512, N=N, K=K, p=4, q=2)
                M, p, q = 512, 4, 2
                a, a_packed, wps, sa, sw = operands(case)
                h = torch.empty((M, N), dtype=torch.float16, device=dev)

                def pack_gemm(i):
                    binding.apmm_pack_activations(a, p, out=a_packed)
                    binding.apmm_gemm(M, N, K, p, q, a_packed, wps[0], want_i32=False, want_f16=True, w_scale=sw,
                                      a_scale=sa, c_f16=h)

                nb = N * K * q / 8.0 + M * K * p / 8.0 + 2.0 * M * N + 2.0 * (M + N) + M * K + M * K * p / 8.0
                tc, tg = clock_calls(pack_gemm, 200), clock_graph(pack_gemm, 10)
                fused_calls += tc
                fused_graph += tg
                row("cfg5 %s: pack + GEMM, fp16" % name, case, tc, tg, nb)
                del a, a_packed, wps
                torch.cuda.empty_cache()
            ops = sum(2.0 * c["M"] * c["N"] * c["K"] for c in inputs.config_cases(5))
            print("| cfg5 whole sweep (7 linears) | | | | W2A4 | %.1f | %.1f | %.0f | | %.1f (int8 MFMA) | %.0f %% |" % (
                sweep_calls, sweep_graph, ops / min(sweep_calls, sweep_graph) / 1e6, ops / INT8_PEAK * 1e6,
                100.0 * ops / INT8_PEAK * 1e6 / min(sweep_calls, sweep_graph)), flush=True)
            print("| cfg5 whole layer, shared inputs fused (4 linears) | | | | W2A4 | %.1f | %.1f | %.0f | | %.1f (int8 MFMA) | %.0f %% |" % (
                fused_calls, fused_graph, ops / min(fused_calls, fused_graph) / 1e6, ops / INT8_PEAK * 1e6,
                100.0 * ops / INT8_PEAK * 1e6 / min(fused_calls, fused_graph)), flush=True)


if __name__ == "__main__":
    main()
