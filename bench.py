#!/usr/bin/env python3
"""Benchmark of the bipolar-INT GEMM hot path on one MI355X.

Default run (the line the driver records).  Workload: the square W1A2 case (M = N = K = 4096, 1-bit
weights, 2-bit activations, int32 output), the shape of the paper's Table 1 on which the headline metric is
quoted.  One step = one pass of the hot path on device-resident inputs: online activation packing (paper
Sec. 4.1) followed by the GEMM with on-chip recovery (paper Sec. 3.2 / 4.2).  The weights are packed once,
outside the timed region, as an inference engine would do.  Prints ONE JSON line:
  value         effective TOPS = 2*M*N*K / step time
  roofline      the dominant kernel (the GEMM): HIP events that ride on the kernel's own dispatch, on the
                stream it is launched on, for every fourth launch of the timed region; the kernel's name is
                what the library reports it launched; `traffic` is read from the kept rocprofv3 counter
                summary under profiles/ when that summary is for the same kernel, else null
  decode        the second half of the metric, measured in the same run: the decode shape M = 1,
                N = 11008, K = 4096 at W2A2, activations as codes (packed inside the one launch), fp16 scale
                epilogue, walking over more than 512 MiB of distinct packed weight copies so that no cache
                serves them: microseconds per call inside a captured graph, GB/s of algorithmic bytes and
                the fraction of the 8 TB/s HBM peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload

Other modes (markdown tables, not the default line):
  --all-configs [--configs 1,2,3,4,5]   every workload configuration against its roofline
  --tile-designs                        large tiles against the K split across the waves of a workgroup, on outputs
                                        of one round of tiles
  --small-m                             1 - 64 tokens over code widths (packed and from codes) and one token over growing
                                        weight matrices
  --decode-designs                      design A (matrix unit) against design B (XOR + popcount) at the decode shape
  --decode-layer                        the seven linears of a decoder layer as seven calls and as one grouped launch
  --paper-shapes                        the shapes of the paper's Tables 1 and 2, GEMM only, and the
                                        Sec. 4.2 ablation (plane pairs to global memory + recovery pass, planes
                                        on the matrix unit with recovery in registers) against the fused kernel
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published dense matrix peaks (TFLOP/s or TOP/s) and HBM bandwidth
PEAK = {"fp4": 10100.0, "int8": 5000.0}   # int8: the peak the problem statement's target is expressed against
HBM_PEAK_GBS = 8000.0
INT8_PEAK = 5.0e15
HBM_PEAK = 8.0e12
PAPER_W1A2_4096_TOPS = 2 * 4096 ** 3 / 160e-6 / 1e12   # paper Table 1: 160 us on an RTX 3090

# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary of this command (with --calibrate-copy); its last lines name
# the kernel it was taken for and the calibrated bytes per launch
TRAFFIC_PROFILE = os.path.join("profiles", "gemm_mfma_fp4_w1a2_4096_hbm_traffic.txt")

ALGOS = {"auto": 0, "valu": 1, "fp4": 4}

# paper Table 1 / Table 2, RTX 3090, microseconds
PAPER_US = {
    ("W1A2", 1024, 1024, 1024): 8.7, ("W1A2", 2048, 2048, 2048): 30.6, ("W1A2", 4096, 4096, 4096): 160.0,
    ("W2A2", 1024, 1024, 1024): 12.0, ("W2A2", 2048, 2048, 2048): 54.8, ("W2A2", 4096, 4096, 4096): 323.0,
    ("W1A2", 1024, 4096, 4096): 51.0, ("W1A2", 1024, 11008, 4096): 129.0, ("W1A2", 1024, 4096, 11008): 109.0,
    ("W2A2", 1024, 4096, 4096): 85.0, ("W2A2", 1024, 11008, 4096): 222.0, ("W2A2", 1024, 4096, 11008): 210.0,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed steps for this long before the warmup steps: after idling the GPU needs about "
                         "40 ms of work before its clocks settle (a step takes 50 us in the first 10 ms, 33 us later)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-shape measurement")
    ap.add_argument("--algo", choices=sorted(ALGOS), default="auto",
                    help="GEMM kernel: auto picks the E2M1 (fp4) MFMA kernel for this workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 64 MiB device copy (reference for HBM byte counters)")
    ap.add_argument("--all-configs", action="store_true", help="time every workload configuration (markdown)")
    ap.add_argument("--configs", default="1,2,3,4,5", help="with --all-configs: which configurations")
    ap.add_argument("--paper-shapes", action="store_true", help="the paper's table shapes and the ablation (markdown)")
    ap.add_argument("--decode-designs", action="store_true",
                    help="the decode shape (M = 1, 11008 x 4096, W2A2, packed activations, cold weights) on both designs: "
                         "matrix-unit small-M kernel and XOR/popcount small-M kernel (one JSON line)")
    ap.add_argument("--tile-designs", action="store_true",
                    help="large tiles against the K split across waves on outputs of one round of tiles (markdown)")
    ap.add_argument("--small-m", action="store_true",
                    help="the small-M path over code widths and weight sizes (markdown)")
    ap.add_argument("--decode-layer", action="store_true",
                    help="the seven linears of a Llama-2-7B decoder layer at 1, 8 and 16 tokens (W2A2, fp16 epilogue, cold "
                         "weights): seven calls, and one grouped launch of seven independent problems (markdown)")
    return ap.parse_args()


def cpu_baseline(case, seed):
    """Time the oracle (as it stands) on a bounded sample of the workload."""
    import oracle
    from paper_2409_17870_amd import inputs
    cores = oracle.num_threads()
    sample_rows = case["M"] if cores >= 16 else case["M"] // 2
    data = inputs.make_case(case, seed)
    a = data["a_codes"][:sample_rows]
    t0 = time.perf_counter()
    oracle.gemm_i64(a, data["w_codes"], case["p"], case["q"])
    dt = time.perf_counter() - t0
    ops = 2.0 * sample_rows * case["N"] * case["K"]
    return {
        "value": ops / dt / 1e12, "unit": "TOPS", "cores": cores, "kind": "oracle",
        "seconds": dt,
        "sample": "first %d of %d activation rows, all %d output channels, full K=%d" %
                  (sample_rows, case["M"], case["N"], case["K"]),
    }


def profiled_traffic(kernel):
    """Calibrated HBM bytes per launch from the kept counter summary, if it was taken for `kernel`."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    try:
        text = open(path).read()
    except OSError:
        return None, None
    k = re.search(r"^kernel:\s*(\S+)\s*$", text, flags=re.M)
    t = re.search(r"^traffic_bytes_per_launch:\s*(\d+)\s*$", text, flags=re.M)
    if not k or not t or k.group(1) != kernel:
        return None, None
    return int(t.group(1)), TRAFFIC_PROFILE


def graph_us_per_call(torch, step, reps, replays=10):
    """`step(i)` for i < reps captured once into a HIP graph; mean time of one step over `replays` replays."""
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        step(0)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            for i in range(reps):
                step(i)
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < 20.0:      # clocks settle
            g.replay()
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (replays * reps)


def decode_leg(torch, binding, inputs):
    """Configuration 3 at M = 1, N = 11008, K = 4096 (W2A2), from codes, cold rotating weights."""
    dev = torch.device("cuda:0")
    M, N, K, p, q = 1, 11008, 4096, 2, 2
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, inputs.BASE_SEED + 3)
    a = torch.from_numpy(data["a_codes"]).to(dev)
    sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
    wp0 = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), q)
    w_bytes = N * K * q / 8.0
    copies = int((512 << 20) // w_bytes) + 2
    wps = [wp0] + [wp0.clone() for _ in range(copies - 1)]
    h = torch.empty((M, N), dtype=torch.float16, device=dev)

    def call(i):
        binding.apmm_gemm_from_codes(a, N, p, q, wps[i % copies], want_i32=False, want_f16=True, w_scale=sw, a_scale=sa,
                                     c_f16=h)

    us_graph = graph_us_per_call(torch, call, copies)
    kernel = binding.apmm_last_gemm_kernel()
    # the kernel alone: events on its own dispatch, eager launches over the same rotating copies
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(2 * copies)]
    for e0, e1 in evs:
        e0.record()
        e1.record()
    torch.cuda.synchronize()
    for i, (e0, e1) in enumerate(evs):
        binding.apmm_time_next_gemm(e0, e1)
        call(i)
    torch.cuda.synchronize()
    kernel_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs[copies:])
    kernel_us = kernel_us[len(kernel_us) // 2]
    nbytes = w_bytes + M * K + 2.0 * M * N + 2.0 * (M + N)      # packed weights + codes + fp16 output + scales
    gbs = nbytes / us_graph / 1e3
    return {
        "workload": "decode W2A2 M=1 N=11008 K=4096, apmm_gemm_from_codes (activation codes packed inside the one "
                    "launch), fp16 scale epilogue, %d distinct packed weight copies (%.0f MiB) in rotation"
                    % (copies, copies * w_bytes / 2 ** 20),
        "kernel": kernel, "us_per_call": us_graph, "timing": "captured HIP graph of %d calls, 10 replays" % copies,
        "kernel_us_median": kernel_us, "algorithmic_bytes": nbytes, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": gbs / HBM_PEAK_GBS, "bound": "hbm",
    }


def decode_designs(args):
    """Design A against design B at the decode shape: apmm_gemm_ex with the two small-M algo ids on the same packed
    operands, each walking over more than 512 MiB of packed weight copies; kernel time from events on the dispatch."""
    import torch
    from paper_2409_17870_amd import binding, inputs
    dev = torch.device("cuda:0")
    M, N, K, p, q = 1, 11008, 4096, 2, 2
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, inputs.BASE_SEED + 3)
    ap = binding.apmm_pack_activations(torch.from_numpy(data["a_codes"]).to(dev), p)
    sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
    wp0 = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), q)
    w_bytes = N * K * q / 8.0
    copies = int((512 << 20) // w_bytes) + 2
    wps = [wp0] + [wp0.clone() for _ in range(copies - 1)]
    h = torch.empty((M, N), dtype=torch.float16, device=dev)
    nbytes = w_bytes + M * K * p / 8.0 + 2.0 * M * N + 2.0 * (M + N)
    out = {"workload": "decode W2A2 M=1 N=11008 K=4096, packed activations, fp16 scale epilogue, %d packed weight copies "
                       "in rotation" % copies, "algorithmic_bytes": nbytes, "designs": {}}
    for name, algo in (("A: E2M1 MFMA 16x16x128", binding.ALGO_DECODE), ("B: XOR + popcount", binding.ALGO_DECODE_VALU)):
        def call(i):
            binding.apmm_gemm(M, N, K, p, q, ap, wps[i % copies], want_i32=False, want_f16=True, w_scale=sw, a_scale=sa,
                              c_f16=h, algo=algo)
        us_graph = graph_us_per_call(torch, call, copies)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(2 * copies)]
        for e0, e1 in evs:
            e0.record()
            e1.record()
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(evs):
            binding.apmm_time_next_gemm(e0, e1)
            call(i)
        torch.cuda.synchronize()
        k_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs[copies:])
        out["designs"][name] = {"kernel": binding.apmm_last_gemm_kernel(), "us_per_call_in_graph": us_graph,
                                "kernel_us_median": k_us[len(k_us) // 2], "GB/s": nbytes / us_graph / 1e3,
                                "frac_of_hbm_peak": nbytes / us_graph / 1e3 / HBM_PEAK_GBS}
    print(json.dumps(out))


def decode_layer(args):
    """Grouped launch (apmm_gemm_grouped) against one call per linear, weights of 14 layers in rotation (672 MiB)."""
    import torch
    from paper_2409_17870_amd import binding
    dev = torch.device("cuda:0")
    p = q = 2
    H, F = 4096, 11008
    shapes = [("q", H, H), ("k", H, H), ("v", H, H), ("o", H, H), ("gate", F, H), ("up", F, H), ("down", H, F)]
    layers = 14
    weights = [{n: binding.apmm_pack_weights(torch.randint(0, 4, (N, K), dtype=torch.uint8, device=dev), q)
                for (n, N, K) in shapes} for _ in range(layers)]
    w_bytes = sum(N * K * q / 8.0 for (_, N, K) in shapes)
    print("| tokens | seven calls from codes (us per layer) | one grouped launch, packed activations (us) | one grouped "
          "launch from codes (us) | grouped: GB/s of weights | of the HBM peak |")
    print("|---|---|---|---|---|---|")
    for M in (1, 8, 16):
        x = {H: torch.randint(0, 4, (M, H), dtype=torch.uint8, device=dev),
             F: torch.randint(0, 4, (M, F), dtype=torch.uint8, device=dev)}
        xp = {K: binding.apmm_pack_activations(x[K], p) for K in x}
        sa = (torch.rand(M, device=dev) * 0.09 + 0.01).half()
        sw = {n: (torch.rand(N, device=dev) * 0.09 + 0.01).half() for (n, N, K) in shapes}
        out = {n: torch.empty((M, N), dtype=torch.float16, device=dev) for (n, N, K) in shapes}

        def calls(i):
            for (n, N, K) in shapes:
                binding.apmm_gemm_from_codes(x[K], N, p, q, weights[i % layers][n], want_i32=False, want_f16=True,
                                             w_scale=sw[n], a_scale=sa, c_f16=out[n])

        def grouped(codes):
            def f(i):
                probs = []
                for (n, N, K) in shapes:
                    d = dict(M=M, N=N, K=K, w_packed=weights[i % layers][n], c_f16=out[n], w_scale=sw[n], a_scale=sa)
                    d["a_codes" if codes else "a_packed"] = x[K] if codes else xp[K]
                    probs.append(d)
                binding.apmm_gemm_grouped(probs, p, q)
            return f

        t_calls = graph_us_per_call(torch, calls, layers)
        t_packed = graph_us_per_call(torch, grouped(False), layers)
        t_codes = graph_us_per_call(torch, grouped(True), layers)
        best = min(t_packed, t_codes)
        print("| %d | %.1f | %.1f | %.1f | %.0f | %.0f %% |" % (M, t_calls, t_packed, t_codes, w_bytes / best / 1e3,
                                                             100.0 * w_bytes / best / 1e3 / HBM_PEAK_GBS), flush=True)


def tile_designs(args):
    """The two tile designs of the matrix-unit GEMM on outputs of one round of tiles: large tiles whose waves own parts
    of the output and sweep all of K (APMM_ALGO_MFMA_FP4), and one tile per workgroup whose four waves split K
    (APMM_ALGO_MFMA_KSPLIT).  GEMM only, fp16 output, inside a captured graph.  Under rocprofv3 the two kernels
    appear under their own names (kernel trace, L1 / L2 request counters)."""
    import torch
    from paper_2409_17870_amd import binding
    dev = torch.device("cuda:0")
    print("| M | N | K | scheme | large tiles (us) | kernel | K split across waves (us) | kernel | AUTO takes |")
    print("|---|---|---|---|---|---|---|---|---|")
    for (M, N, K, p, q) in ((512, 5120, 5120, 4, 2), (512, 5120, 13824, 4, 2), (512, 4096, 4096, 2, 2), (512, 4096, 11008, 2, 2),
                            (128, 4096, 4096, 2, 2), (256, 4096, 11008, 2, 1)):
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        ap, wp = binding.apmm_pack_activations(a, p), binding.apmm_pack_weights(w, q)
        sa = (torch.rand(M, device=dev) * 0.09 + 0.01).half()
        sw = (torch.rand(N, device=dev) * 0.09 + 0.01).half()
        h = torch.empty((M, N), dtype=torch.float16, device=dev)
        cells = []
        for algo in (binding.ALGO_MFMA_FP4, binding.ALGO_MFMA_KSPLIT, binding.ALGO_AUTO):
            def call(i):
                binding.apmm_gemm(M, N, K, p, q, ap, wp, want_i32=False, want_f16=True, w_scale=sw, a_scale=sa, c_f16=h,
                                  algo=algo)
            for i in range(200):   # settle the clocks on this kernel
                call(i)
            us = graph_us_per_call(torch, call, 20)
            cells.append((us, binding.apmm_last_gemm_kernel()))
        print("| %d | %d | %d | W%dA%d | %.1f | %s | %.1f | %s | %s |" % (M, N, K, q, p, cells[0][0], cells[0][1], cells[1][0],
                                                                  cells[1][1], cells[2][1]))


def small_m(args):
    """The small-M path over code widths and weight sizes.  First table: 1 / 16 / 64 tokens at 4096 x 4096 and
    11008 x 4096 for several schemes, packed activations and from codes, whatever kernel AUTO takes.  Second table: one
    token at W2A2 from codes over growing weight matrices.  Weights rotate over more than 512 MiB of packed copies;
    microseconds per call inside a captured graph."""
    import torch
    from paper_2409_17870_amd import binding
    dev = torch.device("cuda:0")

    def timed(M, N, K, p, q, codes):
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        wp0 = binding.apmm_pack_weights(torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev), q)
        copies = int((512 << 20) // (N * K * q / 8.0)) + 2
        wps = [wp0] + [wp0.clone() for _ in range(copies - 1)]
        ap = binding.apmm_pack_activations(a, p)
        ws = torch.empty(binding.apmm_packed_activation_bytes(M, K, p), dtype=torch.uint8, device=dev)
        sa = (torch.rand(M, device=dev) * 0.09 + 0.01).half()
        sw = (torch.rand(N, device=dev) * 0.09 + 0.01).half()
        h = torch.empty((M, N), dtype=torch.float16, device=dev)

        def call(i):
            if codes:
                binding.apmm_gemm_from_codes(a, N, p, q, wps[i % copies], want_i32=False, want_f16=True, w_scale=sw,
                                             a_scale=sa, c_f16=h, workspace=ws)
            else:
                binding.apmm_gemm(M, N, K, p, q, ap, wps[i % copies], want_i32=False, want_f16=True, w_scale=sw,
                                  a_scale=sa, c_f16=h)
        for i in range(copies):
            call(i)
        return graph_us_per_call(torch, call, copies), binding.apmm_last_gemm_kernel()

    print("| scheme | N | K | tokens | packed (us) | kernel | from codes (us) | kernel (the last one, when a packing launch precedes it) |")
    print("|---|---|---|---|---|---|---|---|")
    for (p, q) in ((2, 2), (2, 4), (4, 2), (4, 4), (1, 1)):
        for (N, K) in ((4096, 4096), (11008, 4096)):
            for M in (1, 16, 64):
                tp, kp = timed(M, N, K, p, q, False)
                tc, kc = timed(M, N, K, p, q, True)
                print("| W%dA%d | %d | %d | %d | %.1f | %s | %.1f | %s |" % (q, p, N, K, M, tp, kp, tc, kc))
    print()
    print("| N | K | packed weights (MiB) | one token, W2A2, from codes (us) | TB/s of weights | of the HBM peak |")
    print("|---|---|---|---|---|---|")
    for (N, K) in ((4096, 4096), (11008, 4096), (32000, 4096), (28672, 8192), (8192, 28672), (128256, 4096)):
        t, _ = timed(1, N, K, 2, 2, True)
        b = N * K * 2 / 8.0
        print("| %d | %d | %.1f | %.1f | %.2f | %.0f %% |" % (N, K, b / 2 ** 20, t, b / t / 1e6, 100 * b / t / 1e6 / 8.0))


def headline(args):
    import torch
    from paper_2409_17870_amd import binding, inputs
    dev = torch.device("cuda:0")

    case = inputs.config_cases(2)[0]
    seed = inputs.BASE_SEED + 2
    M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
    data = inputs.make_case(case, seed)
    a_codes = torch.from_numpy(data["a_codes"]).to(dev)
    w_codes = torch.from_numpy(data["w_codes"]).to(dev)
    w_packed = binding.apmm_pack_weights(w_codes, q)            # offline
    a_packed = torch.empty(binding.apmm_packed_activation_bytes(M, K, p), dtype=torch.uint8, device=dev)
    c = torch.empty((M, N), dtype=torch.int32, device=dev)
    algo = ALGOS[args.algo]

    def step(events=None):
        binding.apmm_pack_activations(a_codes, p, out=a_packed)
        if events is not None:
            # the two HIP events ride on the GEMM kernel's own dispatch (hipExtLaunchKernel) on the stream
            # the kernel is launched on: they hold the kernel's begin and end, without dispatch gaps
            binding.apmm_time_next_gemm(events[0], events[1])
        binding.apmm_gemm(M, N, K, p, q, a_packed, w_packed, c_i32=c, algo=algo)

    # every EVENT_EVERY-th GEMM launch of the timed region carries a pair of HIP events
    EVENT_EVERY = 4

    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           if i % EVENT_EVERY == 0 and args.algo != "valu" else None for i in range(args.steps)]
    for pair in evs:
        if pair is not None:       # a first record creates the event handles
            pair[0].record()
            pair[1].record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel = binding.apmm_last_gemm_kernel()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    brackets = [e for e in evs if e is not None]
    if brackets:
        gemm_ms = sum(e0.elapsed_time(e1) for e0, e1 in brackets) / len(brackets)
    else:                          # the XOR/popcount kernel takes no timing events: whole step minus nothing
        gemm_ms = ms_per_step
    ops = 2.0 * M * N * K
    value = ops / (ms_per_step * 1e-3) / 1e12
    achieved = ops / (gemm_ms * 1e-3) / 1e12

    mfma = kernel.startswith("gemm_mfma_direct_kernel")
    operand = "fp4" if mfma else "int8"
    traffic, traffic_source = profiled_traffic(kernel)
    if mfma:
        bound, peak = "mfma", PEAK[operand]
    else:
        # XOR/popcount kernel: one XOR, one popcount and one shift-and-add per output, plane pair and 16 elements on
        # the vector ALU: 256 CUs x 64 lanes x 2.4 GHz integer operations per second
        bound, peak = "alu", 2.0 * 16 / (3.0 * p * q) * 256 * 64 * 2.4e9 / 1e12
    out = {
        "metric": "effective TOPS (2*M*N*K/s), W1A2 bipolar-INT GEMM 4096^3 (activation pack + GEMM); "
                  "GB/s at M=1 decode in `decode`",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_ms": args.settle_ms, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": value / PAPER_W1A2_4096_TOPS,
        "baseline_note": "paper Table 1: 160 us = %.0f effective TOPS on an NVIDIA RTX 3090 (GEMM only)"
                         % PAPER_W1A2_4096_TOPS,
        "dtype": "fp4" if mfma else "u32",
        "dtype_note": "E2M1 MFMA operands recombined from bit planes, fp32 accumulate that is exact for this path"
                      if mfma else "XOR + popcount on 32-bit words",
        "data": "synthetic",
        "config": {"workload": "square W1A2 GEMM M=N=K=4096, Bernoulli(1/2) bits, int32 output",
                   "M": M, "N": N, "K": K, "weight_bits": q, "activation_bits": p,
                   "step": "apmm_pack_activations + apmm_gemm, weights pre-packed", "algo": args.algo},
        "gemm_ms": gemm_ms, "pack_ms": ms_per_step - gemm_ms,
        "roofline": {"bound": bound, "kernel": kernel,
                     "achieved": achieved, "peak": peak, "unit": "TOP/s",
                     "frac": achieved / peak,
                     "frac_of_int8_peak": achieved / PEAK["int8"],
                     "launches_timed": len(brackets),
                     "traffic": traffic, "traffic_source": traffic_source},
    }
    del a_codes, w_codes, w_packed, a_packed, c
    torch.cuda.empty_cache()
    if not args.no_decode:
        out["decode"] = decode_leg(torch, binding, inputs)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case, seed)
    print(json.dumps(out))


# ----------------------------------------------------------------------------------------------------------
# --all-configs: every workload configuration of the problem statement against its roofline.
#
# Step of a configuration (what is inside the timed region):
#   1, 2   GEMM with int32 output, and activation packing + GEMM
#   3      decode shapes: GEMM straight from the activation codes (the online packing is part of the call), fp16
#          output through the scale epilogue; weights pre-packed
#   4      GEMM with int32 and fp16 outputs (activations pre-packed), and with the packing
#   5      activation packing + GEMM with the fp16 epilogue, per linear and for the whole decoder-layer sweep
# Two clocks per step: "calls" is a HIP event pair around a loop of back-to-back calls through the C ABI (the host's
# launch cost is inside; for steps of a few microseconds that is all one sees), "graph" is the same loop captured
# once into a HIP graph and replayed (what a serving loop that captures its decode step pays).  For the HBM-bound
# decode shapes the loop walks over enough distinct packed weight copies (640 MiB) that neither L2 nor the
# memory-side cache serves them.
# Roofline: t_roof = max(2 M N K / 5.0 POP/s, algorithmic bytes / 8 TB/s); bytes = packed weights + packed
# activations + outputs (+ the unpacked codes read and the packed activations written when packing is inside the
# step).  Integer GEMM time does not depend on the values, so codes are random; parity on these shapes is the
# tests' job.
# ----------------------------------------------------------------------------------------------------------
def all_configs(args):
    import torch
    from paper_2409_17870_amd import binding, inputs
    dev = torch.device("cuda:0")

    def settle(step, ms=40.0):
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

    def clock_graph(step, reps):
        return graph_us_per_call(torch, step, reps)

    def row(label, case, us_calls, us_graph, nbytes):
        M, N, K = case["M"], case["N"], case["K"]
        ops = 2.0 * M * N * K
        t_roof = max(ops / INT8_PEAK, nbytes / HBM_PEAK) * 1e6
        bound = "int8 MFMA" if ops / INT8_PEAK > nbytes / HBM_PEAK else "HBM"
        best = min(us_calls, us_graph)
        print("| %s | %d | %d | %d | W%dA%d | %.1f | %.1f | %.0f | %.0f | %.2f (%s) | %.0f %% | %s |" % (
            label, M, N, K, case["q"], case["p"], us_calls, us_graph, ops / best / 1e6, nbytes / best / 1e3,
            t_roof, bound, 100.0 * t_roof / best, binding.apmm_last_gemm_kernel()), flush=True)

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

    print("| step | M | N | K | scheme | calls (us) | graph (us) | eff. TOPS | GB/s | t_roof us (bound) | of roofline | GEMM kernel |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|")
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
            print("| cfg5 whole sweep (7 linears) | | | | W2A4 | %.1f | %.1f | %.0f | | %.1f (int8 MFMA) | %.0f %% | |" % (
                sweep_calls, sweep_graph, ops / min(sweep_calls, sweep_graph) / 1e6, ops / INT8_PEAK * 1e6,
                100.0 * ops / INT8_PEAK * 1e6 / min(sweep_calls, sweep_graph)), flush=True)
            print("| cfg5 whole layer, shared inputs fused (4 linears) | | | | W2A4 | %.1f | %.1f | %.0f | | %.1f (int8 MFMA) | %.0f %% | |" % (
                fused_calls, fused_graph, ops / min(fused_calls, fused_graph) / 1e6, ops / INT8_PEAK * 1e6,
                100.0 * ops / INT8_PEAK * 1e6 / min(fused_calls, fused_graph)), flush=True)


# ----------------------------------------------------------------------------------------------------------
# --paper-shapes: GEMM-only times of the shapes of the paper's Table 1 (square MatMuls) and Table 2 (Llama-2-7B
# linear shapes at M = 1024) for W1A2 and W2A2, next to the latencies the paper prints for an RTX 3090.
# ----------------------------------------------------------------------------------------------------------
def paper_shapes(args):
    import torch
    from paper_2409_17870_amd import binding
    dev = torch.device("cuda:0")

    print("| scheme | M | N | K | this library, MI355X: calls (us) | graph (us) | effective TOPS | paper, RTX 3090 (us) |")
    print("|---|---|---|---|---|---|---|---|")
    for (name, M, N, K), paper in PAPER_US.items():
        q, p = int(name[1]), int(name[3])
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        ap, wp = binding.apmm_pack_activations(a, p), binding.apmm_pack_weights(w, q)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)

        def gemm(i):
            binding.apmm_gemm(M, N, K, p, q, ap, wp, c_i32=c)

        for _ in range(200):
            gemm(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            gemm(0)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 200
        ug = graph_us_per_call(torch, gemm, 20)
        print("| %s | %d | %d | %d | %.1f | %.1f | %.0f | %.1f |" % (name, M, N, K, us, ug, 2.0 * M * N * K / min(us, ug) / 1e6, paper),
              flush=True)

    # Ablation for the claim of paper Sec. 4.2, all three schemes as kernels of this library (apmm_gemm_ex algo ids):
    # the fused kernel (recovery moved in front of the multiplier), the planes as +-1 operands on the matrix unit with
    # an accumulator per plane pair and shift-and-add in registers, and the scheme the paper argues against: one
    # plane pair per workgroup, its 32-bit product to global memory, then a shift-and-add pass over those products.
    print()
    print("| scheme (4096^3, int32 out) | fused kernel (us) | planes on the matrix unit, recovery in registers (us) | "
          "plane pairs to global memory + recovery pass (us) | naive / fused |")
    print("|---|---|---|---|---|")
    M = N = K = 4096
    for (p, q) in ((1, 1), (2, 1), (2, 2)):
        a = torch.randint(0, 1 << p, (M, K), dtype=torch.uint8, device=dev)
        w = torch.randint(0, 1 << q, (N, K), dtype=torch.uint8, device=dev)
        ap, wp = binding.apmm_pack_activations(a, p), binding.apmm_pack_weights(w, q)
        c = torch.empty((M, N), dtype=torch.int32, device=dev)
        ws = torch.empty(p * q * M * N * 4, dtype=torch.uint8, device=dev)
        times = []
        for algo, workspace in ((binding.ALGO_AUTO, None), (binding.ALGO_PLANES_REGISTERS, None),
                                (binding.ALGO_PLANE_PAIRS_GLOBAL, ws)):
            def gemm(i):
                binding.apmm_gemm(M, N, K, p, q, ap, wp, c_i32=c, workspace=workspace, algo=algo)
            times.append(graph_us_per_call(torch, gemm, 10))
        print("| W%dA%d | %.1f | %.1f | %.1f | %.1fx |" % (q, p, times[0], times[1], times[2], times[2] / times[0]), flush=True)
        del ws
        torch.cuda.empty_cache()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus %d refused)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2409_17870_amd import binding
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    binding.load()
    if args.all_configs:
        all_configs(args)
    elif args.paper_shapes:
        paper_shapes(args)
    elif args.decode_designs:
        decode_designs(args)
    elif args.tile_designs:
        tile_designs(args)
    elif args.small_m:
        small_m(args)
    elif args.decode_layer:
        decode_layer(args)
    else:
        headline(args)


if __name__ == "__main__":
    main()
