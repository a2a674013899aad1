"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Integer outputs must be bit-exact.  The fp16 epilogue must be within 1e-3 relative
(+1e-6 absolute) of the oracle's double-precision product, the tolerance the problem
statement fixes (one fp32 product chain plus one rounding to binary16 is <= 2^-11 + a few
2^-24 relative).
"""
import numpy as np
import pytest

from paper_2409_17870_amd import inputs

pytestmark = pytest.mark.gpu

VALU, DECODE, FP4, DECODE_VALU, KSPLIT = 1, 3, 4, 5, 8


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2409_17870_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()          # fails loudly if the HIP library is missing
    return torch, binding


def run_case(gpu, data, case, algo=0, want_i32=True, want_f16=None):
    torch, binding = gpu
    dev = torch.device("cuda:0")
    M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
    a = torch.from_numpy(data["a_codes"]).to(dev)
    w = torch.from_numpy(data["w_codes"]).to(dev)
    sa = torch.from_numpy(data["a_scale"]).to(dev) if data["a_scale"] is not None else None
    sw = torch.from_numpy(data["w_scale"]).to(dev) if data["w_scale"] is not None else None
    if want_f16 is None:
        want_f16 = sa is not None or sw is not None
    wp = binding.apmm_pack_weights(w, q)
    ap = binding.apmm_pack_activations(a, p)
    c32, c16 = binding.apmm_gemm(M, N, K, p, q, ap, wp, want_i32=want_i32, want_f16=want_f16,
                                 w_scale=sw, a_scale=sa, algo=algo)
    torch.cuda.synchronize()
    return (c32.cpu().numpy() if c32 is not None else None,
            c16.cpu().numpy() if c16 is not None else None)


def check_f16(got_f16, want_i64, data, oracle):
    sa = data["a_scale"].view(np.uint16) if data["a_scale"] is not None else None
    sw = data["w_scale"].view(np.uint16) if data["w_scale"] is not None else None
    f = oracle.scale_f64(want_i64, sa, sw)
    got = got_f16.astype(np.float64)
    assert np.all(np.abs(got - f) <= 1e-3 * np.abs(f) + 1e-6)


def algos_for(case):
    algos = [VALU]
    if case["p"] <= 4 and case["q"] <= 4:
        algos.append(FP4)
    if (case["M"] <= 16 and case["q"] <= 4 and case["p"] not in (3, 4)) or \
            (case["M"] <= 64 and case["p"] <= 2 and case["q"] <= 2):
        algos.append(DECODE)
    if case["M"] <= 16 and case["q"] <= 4 and case["p"] not in (3, 4):
        algos.append(DECODE_VALU)
    return algos + [0]


# ------------------------------------------------------------- pack layout --
@pytest.mark.parametrize("rows,K,bits", [(1, 1, 1), (5, 31, 3), (32, 128, 2), (33, 129, 4), (70, 500, 8),
                                         (16, 512, 2), (100, 4096, 1), (257, 1000, 5), (37, 4097, 2), (5, 11008, 4),
                                         (3, 20000, 3), (40, 16400, 1), (9, 70000, 7)])
def test_pack_unpack_roundtrip(gpu, rows, K, bits):
    """Includes rows of more than 4096 elements, which four waves share, and the code sums behind the tiles."""
    torch, binding = gpu
    rng = np.random.default_rng(rows * 7919 + K * 13 + bits)
    codes = rng.integers(0, 256, size=(rows, K), dtype=np.uint8)     # high bits are dirt
    dev_codes = torch.from_numpy(codes).to("cuda:0")
    for pack, size, unpack in ((binding.apmm_pack_weights, binding.apmm_packed_bytes, binding.apmm_unpack),
                               (binding.apmm_pack_activations, binding.apmm_packed_activation_bytes,
                                binding.apmm_unpack_activations)):
        packed = pack(dev_codes, bits)
        assert packed.numel() == size(rows, K, bits)
        back = unpack(packed, rows, K, bits).cpu().numpy()
        assert np.array_equal(back, codes & ((1 << bits) - 1))
        # one int32 per padded row at the end of the buffer: the sum of the row's codes over the padded K
        rows_p, k_p = -(-rows // 32) * 32, -(-K // 512) * 512
        sums = packed.cpu().numpy()[-4 * rows_p:].view(np.int32)
        want = (codes & ((1 << bits) - 1)).astype(np.int64).sum(axis=1) + (k_p - K) * ((1 << bits) - 1)
        assert np.array_equal(sums[:rows].astype(np.int64), want) and not sums[rows:].any()


def test_pack_is_plane_decomposition(gpu):
    """Sec. 4.1: the packed buffer holds exactly `bits` one-bit planes (popcount per plane matches).

    Planes 0 and 1 share the words of slots 0 and 1 (even / odd bit positions), plane 2 has slot 2."""
    torch, binding = gpu
    rows, K, bits = 32, 128, 3                                        # K is padded to 512: four tiles
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 8, size=(rows, K), dtype=np.uint8)
    packed = binding.apmm_pack_weights(torch.from_numpy(codes).to("cuda:0"), bits).cpu().numpy()
    sums = packed.view(np.int32)[-rows:]                             # behind the planes: code sum per row
    words = packed.view(np.uint32)[:-rows].reshape(4, bits, rows, 4)[0]  # first tile: [slot][row][word]
    for r in range(rows):
        ones = [sum(bin(int(x) & 0x55555555).count("1") for x in words[0:2, r].ravel()),
                sum(bin(int(x) & 0xAAAAAAAA).count("1") for x in words[0:2, r].ravel()),
                sum(bin(int(x)).count("1") for x in words[2, r])]
        for i in range(bits):
            assert ones[i] == int(((codes[r] >> i) & 1).sum())
    pad = 512 - K                                                     # padded positions hold the all-ones code
    assert np.array_equal(sums, codes.astype(np.int64).sum(axis=1) + pad * ((1 << bits) - 1))


# ------------------------------------------------------------- small cases --
def test_config1_tiny_w1a2(gpu, oracle):
    case = inputs.config_cases(1)[0]
    data = inputs.make_case(case, inputs.BASE_SEED + 1)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], case["p"], case["q"])
    for algo in algos_for(case):
        c32, _ = run_case(gpu, data, case, algo=algo)
        assert c32.dtype == np.int32
        assert np.array_equal(c32.astype(np.int64), want), "algo %d" % algo


@pytest.mark.parametrize("p,q", [(p, q) for p in range(1, 5) for q in range(1, 5)])
def test_all_precisions_several_tiles_ragged(gpu, oracle, p, q):
    """Shapes spanning several workgroup tiles with ragged M, N and K tails."""
    for (M, N, K) in [(150, 300, 384), (70, 45, 200), (300, 520, 130)]:
        case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
        data = inputs.make_case(case, 1000 + 17 * p + q)
        want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
        for algo in algos_for(case):
            c32, c16 = run_case(gpu, data, case, algo=algo)
            assert np.array_equal(c32.astype(np.int64), want), "algo %d shape %s" % (algo, (M, N, K))
            check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (2, 2), (1, 3), (2, 4), (1, 2)])
def test_ablation_plane_schemes(gpu, oracle, p, q):
    """Sec. 4.2 ablation kernels through apmm_gemm_ex: every plane pair's product to global memory plus a recovery
    pass (algo 6, with its workspace), and the planes on the matrix unit with shift-and-add in registers (algo 7);
    several tiles, ragged M, N and K, int32 and fp16 outputs against the oracle."""
    torch, binding = gpu
    for (M, N, K) in [(150, 300, 384), (300, 520, 130), (70, 45, 1100), (256, 128, 512)]:
        case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
        data = inputs.make_case(case, 1500 + 17 * p + q)
        want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
        dev = torch.device("cuda:0")
        ap = binding.apmm_pack_activations(torch.from_numpy(data["a_codes"]).to(dev), p)
        wp = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), q)
        sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
        ws = torch.empty(p * q * M * N * 4, dtype=torch.uint8, device=dev)
        for algo, workspace in ((binding.ALGO_PLANE_PAIRS_GLOBAL, ws), (binding.ALGO_PLANES_REGISTERS, None)):
            c32, c16 = binding.apmm_gemm(M, N, K, p, q, ap, wp, want_i32=True, want_f16=True, w_scale=sw, a_scale=sa,
                                         workspace=workspace, algo=algo)
            torch.cuda.synchronize()
            assert np.array_equal(c32.cpu().numpy().astype(np.int64), want), (algo, M, N, K)
            check_f16(c16.cpu().numpy(), want, data, oracle)
        with pytest.raises(binding.ApmmError) as err:                      # the naive scheme without its workspace
            binding.apmm_gemm(M, N, K, p, q, ap, wp, algo=binding.ALGO_PLANE_PAIRS_GLOBAL, workspace=ws[:-16])
        assert err.value.status == 4


def test_ablation_kernels_decline_wide_activations(gpu):
    torch, binding = gpu
    dev = torch.device("cuda:0")
    a = torch.zeros((64, 256), dtype=torch.uint8, device=dev)
    ap, wp = binding.apmm_pack_activations(a, 4), binding.apmm_pack_weights(a, 2)
    for algo in (binding.ALGO_PLANE_PAIRS_GLOBAL, binding.ALGO_PLANES_REGISTERS):
        with pytest.raises(binding.ApmmError) as err:
            binding.apmm_gemm(64, 64, 256, 4, 2, ap, wp, algo=algo)
        assert err.value.status == 2


@pytest.mark.parametrize("p,q", [(8, 8), (5, 7), (8, 1), (1, 6), (7, 3)])
def test_wide_codes(gpu, oracle, p, q):
    case = dict(M=37, N=50, K=333, p=p, q=q, a_dist="bernoulli", scaled=False)
    data = inputs.make_case(case, 2000 + 17 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, _ = run_case(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)


@pytest.mark.parametrize("p,q", [(3, 3), (4, 4), (4, 1), (3, 2), (4, 2), (3, 1)])
@pytest.mark.parametrize("M", [1, 7, 16, 17, 32, 33, 50, 64, 65])
def test_few_tokens_with_field_form_activations(gpu, oracle, M, p, q):
    """3- and 4-bit activations (field form).  The small-M matrix-unit kernel takes the packed 6-bit fields as its E2M3
    operand for up to 64 tokens (two groups of 32 from 33 on), with weights of one or two plane groups; more tokens
    and the XOR/popcount small-M kernel decline, and automatic selection serves every case."""
    torch, binding = gpu
    case = dict(M=M, N=203, K=1100, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 5500 + 100 * M + 10 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    if M <= 64:
        c32, c16 = run_case(gpu, data, case, algo=DECODE)
        assert binding.apmm_last_gemm_kernel().startswith("gemm_decode_mfma_kernel<%d,%d" % (p, q))
        assert np.array_equal(c32.astype(np.int64), want)
        check_f16(c16, want, data, oracle)
    else:
        with pytest.raises(binding.ApmmError):
            run_case(gpu, data, case, algo=DECODE)
    with pytest.raises(binding.ApmmError):
        run_case(gpu, data, case, algo=DECODE_VALU)
    c32, c16 = run_case(gpu, data, case, algo=0)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,N,K,p,q", [(1, 4096, 4096, 4, 2), (16, 11008, 4096, 4, 1), (32, 4096, 11008, 3, 2), (8, 300, 20000, 4, 2),
                                       (64, 4096, 4096, 4, 2), (40, 5120, 5120, 4, 1)])
def test_small_m_kernel_field_form_llm_shapes(gpu, oracle, M, N, K, p, q):
    """The small-M kernel on packed 3- and 4-bit activations at decode shapes (one and two channel tiles per workgroup,
    several k iterations per wave, K beyond 16384), through apmm_gemm and through apmm_gemm_from_codes with a workspace."""
    from paper_2409_17870_amd import binding
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="normal" if p == 4 else "bernoulli", scaled=True)
    data = inputs.make_case(case, 5600 + M + p)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, c16 = run_case(gpu, data, case, want_i32=True, want_f16=True)
    assert binding.apmm_last_gemm_kernel().startswith("gemm_decode_mfma_kernel")
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)
    c32, c16 = run_from_codes(gpu, data, case, workspace=True)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (5, 3), (2, 4), (8, 2), (1, 4), (6, 4)])
@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 13, 16])
def test_decode_kernel_all_token_counts(gpu, oracle, M, p, q):
    """Small-M kernel: every token-count bucket, ragged N and K, odd plane counts."""
    case = dict(M=M, N=203, K=1100, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 5000 + 100 * M + 10 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    for algo in (DECODE, DECODE_VALU):          # the matrix-unit kernel where it covers the widths, and XOR/popcount
        c32, c16 = run_case(gpu, data, case, algo=algo)
        assert np.array_equal(c32.astype(np.int64), want)
        check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (1, 2), (2, 2)])
@pytest.mark.parametrize("M", [17, 24, 32, 33, 50, 64])
def test_decode_kernel_token_tiles(gpu, oracle, M, p, q):
    """Matrix-unit small-M kernel with two and four tiles of 16 tokens."""
    case = dict(M=M, N=203, K=1100, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 5700 + 100 * M + 10 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    for algo in (DECODE, 0):
        c32, c16 = run_case(gpu, data, case, algo=algo)
        assert np.array_equal(c32.astype(np.int64), want)
        check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M", [5, 40])
def test_decode_kernel_two_row_tiles_per_workgroup(gpu, oracle, M):
    """Enough output channels for the variant whose workgroups own 32 channels; ragged N."""
    case = dict(M=M, N=16421, K=300, p=2, q=2, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 5900 + M)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 2)
    c32, c16 = run_case(gpu, data, case, algo=DECODE)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


def run_from_codes(gpu, data, case, dirty_high_bits=False, workspace=False):
    torch, binding = gpu
    dev = torch.device("cuda:0")
    p, q = case["p"], case["q"]
    a_np = data["a_codes"]
    if dirty_high_bits and p < 8:  # bits above p must be ignored
        a_np = a_np | np.uint8((0xff << p) & 0xff)
    a = torch.from_numpy(a_np).to(dev)
    w = torch.from_numpy(data["w_codes"]).to(dev)
    sa = torch.from_numpy(data["a_scale"]).to(dev) if data["a_scale"] is not None else None
    sw = torch.from_numpy(data["w_scale"]).to(dev) if data["w_scale"] is not None else None
    wp = binding.apmm_pack_weights(w, q)
    ws = None
    if workspace:
        ws = torch.empty(binding.apmm_packed_activation_bytes(case["M"], case["K"], p), dtype=torch.uint8, device=dev)
    c32, c16 = binding.apmm_gemm_from_codes(a, case["N"], p, q, wp, want_i32=True, want_f16=True, w_scale=sw, a_scale=sa,
                                            workspace=ws)
    torch.cuda.synchronize()
    return c32.cpu().numpy(), c16.cpu().numpy()


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (1, 2), (2, 2), (5, 3), (2, 4), (8, 2), (1, 4), (6, 4), (4, 2), (3, 1), (4, 4), (3, 3)])
@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 13, 16])
def test_gemm_from_codes_few_tokens(gpu, oracle, M, p, q):
    """GEMM straight from the activation codes, both small-M kernels, ragged N and K (K = 1100 is neither a
    multiple of 32 nor of 16: whole groups, a partial group and padded groups all occur)."""
    case = dict(M=M, N=203, K=1100, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 6100 + 100 * M + 10 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, c16 = run_from_codes(gpu, data, case, dirty_high_bits=(M % 2 == 1))
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 1), (1, 2), (2, 2), (2, 4), (1, 3), (2, 3), (1, 4), (4, 2), (3, 4), (4, 1)])
@pytest.mark.parametrize("M,N,K", [(17, 203, 1100), (32, 64, 4096), (50, 203, 1111), (64, 16421, 300), (5, 16421, 300), (2, 300, 4096)])
def test_gemm_from_codes_token_tiles(gpu, oracle, M, N, K, p, q):
    """The same on the matrix-unit small-M kernel with one, two and four token tiles and both row-tile counts."""
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 6900 + M + 10 * p + q)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    # (3- and 4-bit activations have the one-launch form up to 32 tokens; beyond, the call needs its workspace)
    c32, c16 = run_from_codes(gpu, data, case, workspace=(p in (3, 4) and M > 32))
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


def test_gemm_from_codes_unaligned_rows_and_refusals(gpu, oracle):
    """Rows that start at odd addresses (K odd) take the byte-wise loads; shapes outside the small-M kernels
    are refused when there is no workspace to pack into, not computed some other way."""
    torch, binding = gpu
    case = dict(M=7, N=90, K=1023, p=2, q=2, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 7001)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 2)
    c32, c16 = run_from_codes(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)
    dev = torch.device("cuda:0")
    for (M, p, q) in ((65, 2, 2), (17, 5, 2), (33, 4, 2), (4, 2, 5)):
        a = torch.zeros((M, 256), dtype=torch.uint8, device=dev)
        wp = binding.apmm_pack_weights(torch.zeros((32, 256), dtype=torch.uint8, device=dev), q)
        with pytest.raises(binding.ApmmError) as err:
            binding.apmm_gemm_from_codes(a, 32, p, q, wp)
        assert err.value.status == 4


@pytest.mark.parametrize("M,N,K,p,q", [(65, 203, 1100, 2, 2), (300, 130, 700, 4, 2), (4, 77, 260, 3, 3), (17, 64, 512, 5, 2),
                                       (16, 8192, 256, 2, 2), (3, 50, 200, 2, 2)])
def test_gemm_from_codes_through_the_workspace(gpu, oracle, M, N, K, p, q):
    """With a workspace every shape is served: packed there and multiplied by the kernel apmm_gemm would take
    (field-form activations, many tokens, wide codes), or still in one launch where that is the faster way."""
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 7100 + M + p)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, c16 = run_from_codes(gpu, data, case, dirty_high_bits=True, workspace=True)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,K,p,q", [(16, 11008, 8, 4), (8, 9000, 8, 2), (13, 20000, 5, 3), (64, 11008, 2, 2),
                                     (33, 20000, 2, 1), (48, 8200, 1, 2), (16, 40000, 2, 2), (2, 70000, 2, 2)])
def test_decode_kernels_with_k_beyond_one_pass(gpu, oracle, M, K, p, q):
    """Activations that do not fit on chip at once: the small-M kernels take K in passes of 32 k blocks (ragged
    last pass), from packed tiles and from codes alike."""
    case = dict(M=M, N=77, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 7300 + M + p)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    for algo in (DECODE, DECODE_VALU) if M <= 16 else (DECODE,):
        c32, c16 = run_case(gpu, data, case, algo=algo)
        assert np.array_equal(c32.astype(np.int64), want)
        check_f16(c16, want, data, oracle)
    c32, c16 = run_from_codes(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 257, 128), (16, 1, 4096), (3, 7, 127), (17, 33, 129)])
def test_degenerate_shapes(gpu, oracle, M, N, K):
    case = dict(M=M, N=N, K=K, p=2, q=2, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 3000 + M + N + K)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 2)
    for algo in algos_for(case):
        c32, c16 = run_case(gpu, data, case, algo=algo)
        assert np.array_equal(c32.astype(np.int64), want), "algo %d" % algo
        check_f16(c16, want, data, oracle)
    c32, c16 = run_from_codes(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q,K", [(2, 1, 2048), (1, 1, 4096), (2, 2, 2560), (2, 1, 3072), (2, 2, 4096), (1, 2, 3500),
                                   (2, 1, 3584)])
def test_two_phase_kernels(gpu, oracle, p, q, K):
    """130 whole 256 x 256 tiles, int32 output only, one sweep of at most 4096 k: the launch rule picks the MFMA
    kernels that store the first part of a tile under the k loop of the second (the uneven cut for 1-bit weights
    from K = 3072 on, else the even one).  Every output against the oracle."""
    case = dict(M=3328, N=2560, K=K, p=p, q=q, a_dist="bernoulli", scaled=False)
    full_check(gpu, oracle, case, 7000 + 10 * p + q)


def test_long_k_beyond_the_fp32_exactness_bound(gpu, oracle):
    """4 K (2^p - 1)(2^q - 1) >= 2^24: the MFMA kernel declines, auto falls back to XOR/popcount."""
    torch, binding = gpu
    case = dict(M=20, N=24, K=20000, p=4, q=4, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 7100)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 4, 4)
    with pytest.raises(binding.ApmmError):
        run_case(gpu, data, case, algo=FP4)
    c32, c16 = run_case(gpu, data, case, algo=0)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,K,p", [(1, 64, 2), (5, 100, 3), (33, 513, 4), (64, 4096, 2), (16, 11008, 4), (7, 250, 1),
                                   (40, 1000, 8)])
def test_quantize_pack_matches_the_oracle(gpu, oracle, M, K, p):
    """Fused quantise + pack of float16 activations: codes and per-token scales bit-exact."""
    torch, binding = gpu
    x = inputs.normal_features_f16(8000 + M + K + p, inputs.TAG_A, M, K, outlier_every=37)
    if M > 3:
        x[3] = 0                                                       # a row of zeros: scale 0, code of +1
    want_codes, want_scale = oracle.quantize_rows(x, p)
    packed, scale = binding.apmm_quantize_pack_activations(torch.from_numpy(x).to("cuda:0"), p)
    codes = binding.apmm_unpack_activations(packed, M, K, p).cpu().numpy()
    assert np.array_equal(scale.cpu().numpy().view(np.uint16), want_scale)
    assert np.array_equal(codes, want_codes)
    # the packed operand is the one apmm_pack_activations gives for those codes (row sums included)
    again = binding.apmm_pack_activations(torch.from_numpy(want_codes).to("cuda:0"), p)
    assert torch.equal(packed, again)


def test_quantized_activations_through_the_gemm(gpu, oracle):
    """float16 activations -> quantise + pack -> GEMM with the fp16 epilogue, against the oracle's
    quantiser, integer GEMM and double-precision scaling."""
    torch, binding = gpu
    M, N, K, p, q = 48, 200, 1024, 4, 2
    x = inputs.normal_features_f16(8100, inputs.TAG_A, M, K, outlier_every=64)
    w = inputs.bernoulli_codes(8100, inputs.TAG_W, N, K, q)
    sw = inputs.scales_f16(8100, inputs.TAG_W_SCALE, N)
    codes, sa_bits = oracle.quantize_rows(x, p)
    want = oracle.gemm_i64(codes, w, p, q)
    ap, sa = binding.apmm_quantize_pack_activations(torch.from_numpy(x).to("cuda:0"), p)
    wp = binding.apmm_pack_weights(torch.from_numpy(w).to("cuda:0"), q)
    c32, c16 = binding.apmm_gemm(M, N, K, p, q, ap, wp, want_i32=True, want_f16=True,
                                 w_scale=torch.from_numpy(sw).to("cuda:0"), a_scale=sa)
    torch.cuda.synchronize()
    assert np.array_equal(c32.cpu().numpy().astype(np.int64), want)
    f = oracle.scale_f64(want, sa_bits, sw.view(np.uint16))
    got = c16.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - f) <= 1e-3 * np.abs(f) + 1e-6)


@pytest.mark.parametrize("p,q", [(2, 2), (2, 4), (4, 2), (3, 3)])
@pytest.mark.parametrize("M", [1, 2, 8, 16, 40])
def test_grouped_launch_matches_single_calls_and_the_oracle(gpu, oracle, M, p, q):
    """q/k/v-like (shared activations) and gate/up-like linears plus some of another K (one of them too long for
    a single on-chip pass at the larger token counts) in one grouped call."""
    torch, binding = gpu
    dev = torch.device("cuda:0")
    long_k = 40000 if p * q <= 4 else 9000   # within the fp32 exactness bound of the matrix-unit kernels for wider codes
    shapes = [(96, 512), (80, 512), (33, 512), (200, 512), (150, 512), (64, 1280), (16, 130), (48, 512), (40, long_k), (24, 512)]
    acts = {}
    problems, wants = [], []
    for i, (N, K) in enumerate(shapes):
        if K not in acts:
            a = inputs.bernoulli_codes(9000 + K, inputs.TAG_A, M, K, p)
            sa = inputs.scales_f16(9000 + K, inputs.TAG_A_SCALE, M)
            a_dev = torch.from_numpy(a).to(dev)
            acts[K] = (a, binding.apmm_pack_activations(a_dev, p), sa, torch.from_numpy(sa).to(dev), a_dev)
        a, ap, sa, sa_dev, a_dev = acts[K]
        w = inputs.bernoulli_codes(9100 + i, inputs.TAG_W, N, K, q)
        sw = inputs.scales_f16(9100 + i, inputs.TAG_W_SCALE, N)
        problems.append(dict(M=M, N=N, K=K, a_packed=ap, a_dev=a_dev,
                             w_packed=binding.apmm_pack_weights(torch.from_numpy(w).to(dev), q),
                             c_i32=torch.zeros((M, N), dtype=torch.int32, device=dev),
                             c_f16=torch.zeros((M, N), dtype=torch.float16, device=dev),
                             w_scale=torch.from_numpy(sw).to(dev), a_scale=sa_dev))
        want = oracle.gemm_i64(a, w, p, q)
        wants.append((want, oracle.scale_f64(want, sa.view(np.uint16), sw.view(np.uint16))))
    binding.apmm_gemm_grouped(problems, p, q)
    torch.cuda.synchronize()
    for pr, (want, f) in zip(problems, wants):
        assert np.array_equal(pr["c_i32"].cpu().numpy().astype(np.int64), want)
        got = pr["c_f16"].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - f) <= 1e-3 * np.abs(f) + 1e-6)
    binding.apmm_gemm_grouped([], p, q)                                 # nothing to do
    if p > 2:
        return   # 3- and 4-bit activations reach the small-M kernels packed only
    # the same list with the activations as unpacked codes (every second entry, so that runs of both kinds form)
    mixed = []
    for i, pr in enumerate(problems):
        e = dict(pr, c_i32=torch.zeros_like(pr["c_i32"]), c_f16=torch.zeros_like(pr["c_f16"]))
        if i % 3 != 2:
            e["a_codes"], e["a_packed"] = pr["a_dev"], None
        mixed.append(e)
    binding.apmm_gemm_grouped(mixed, p, q)
    torch.cuda.synchronize()
    for pr, (want, f) in zip(mixed, wants):
        assert np.array_equal(pr["c_i32"].cpu().numpy().astype(np.int64), want)
        got = pr["c_f16"].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - f) <= 1e-3 * np.abs(f) + 1e-6)


def test_extreme_values_hit_the_bound(gpu, oracle):
    """All-ones x all-ones and all-ones x all-zeros reach +-K(2^p-1)(2^q-1)."""
    torch, binding = gpu
    M, N, K, p, q = 40, 40, 4096, 4, 4
    a = np.full((M, K), 15, dtype=np.uint8)
    w = np.full((N, K), 15, dtype=np.uint8)
    w[::2] = 0
    data = dict(a_codes=a, w_codes=w, a_scale=None, w_scale=None)
    want = oracle.gemm_i64(a, w, p, q)
    assert want.max() == K * 225 and want.min() == -K * 225
    for algo in (VALU, FP4, 0):
        c32, _ = run_case(gpu, data, dict(M=M, N=N, K=K, p=p, q=q), algo=algo)
        assert np.array_equal(c32.astype(np.int64), want)


def test_empty_problem_and_outputs_selection(gpu, oracle):
    torch, binding = gpu
    case = dict(M=20, N=24, K=256, p=2, q=1, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 4000)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 1)
    c32, c16 = run_case(gpu, data, case, want_i32=False, want_f16=True)
    assert c32 is None
    check_f16(c16, want, data, oracle)
    # fp16 output without scales is a plain conversion (values here are exactly representable)
    plain = dict(data, a_scale=None, w_scale=None)
    c32, c16 = run_case(gpu, plain, case, want_i32=True, want_f16=True)
    assert np.array_equal(c16.astype(np.int64), want)
    # M == 0: nothing to do
    empty = torch.empty((0, 24), dtype=torch.int32, device="cuda:0")
    wp = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to("cuda:0"), 1)
    binding.apmm_gemm(0, 24, 256, 2, 1, wp, wp, c_i32=empty)


@pytest.mark.parametrize("M", [1, 7, 40, 300])
@pytest.mark.parametrize("which", ["a_scale", "w_scale"])
def test_one_scale_vector_only(gpu, oracle, M, which):
    """Only one of the two scale vectors: the missing one counts as 1 (small-M kernels, both tile kernels,
    fp16 alone and next to int32, packed activations and codes)."""
    case = dict(M=M, N=130, K=640, p=2, q=2, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 4100 + M)
    one = dict(data, a_scale=data["a_scale"] if which == "a_scale" else None,
               w_scale=data["w_scale"] if which == "w_scale" else None)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 2)
    for want_i32 in (True, False):
        c32, c16 = run_case(gpu, one, case, want_i32=want_i32, want_f16=True)
        check_f16(c16, want, one, oracle)
        if want_i32:
            assert np.array_equal(c32.astype(np.int64), want)
    c32, c16 = run_from_codes(gpu, one, case, workspace=True)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, one, oracle)


@pytest.mark.parametrize("M,N,K,p,q", [(2, 150000, 128, 1, 1), (16, 70001, 200, 2, 2), (70001, 48, 128, 2, 1),
                                       (1048600, 8, 64, 5, 1), (40, 33000, 100, 2, 2)])
def test_long_dimensions(gpu, oracle, M, N, K, p, q):
    """Many output channels for the small-M kernels (tens of thousands of workgroups), many rows for the tile
    kernels and for the general kernel (whose grid used to end at about a million rows)."""
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=False)
    data = inputs.make_case(case, 4300 + p)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, _ = run_case(gpu, data, case, want_f16=False)
    assert np.array_equal(c32.astype(np.int64), want)


def test_seeded_random_shapes_every_entry_point(gpu, oracle):
    """Sixty shapes and widths drawn from a fixed seed (token counts around the kernels' thresholds, ragged N and K):
    apmm_gemm with automatic kernel choice and apmm_gemm_from_codes against the oracle."""
    rng = np.random.default_rng(20240917)
    for i in range(60):
        M = int(rng.choice([1, 2, 3, 7, 15, 16, 17, 31, 33, 63, 64, 65, 100, 257]))
        N = int(rng.integers(1, 400))
        K = int(rng.choice([1, 31, 64, 127, 128, 500, 512, 513, 1100, 2049, 4100]))
        p, q = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
        data = inputs.make_case(case, 8000 + i)
        want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
        c32, c16 = run_case(gpu, data, case)
        assert np.array_equal(c32.astype(np.int64), want), case
        check_f16(c16, want, data, oracle)
        c32, c16 = run_from_codes(gpu, data, case, dirty_high_bits=bool(i & 1), workspace=True)
        assert np.array_equal(c32.astype(np.int64), want), case
        check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,p,q", [(3, 8, 8), (40, 7, 8), (200, 8, 6), (300, 4, 4)])
def test_fp16_output_beyond_the_binary16_range(gpu, oracle, M, p, q):
    """Wide codes with only one scale vector: many products leave the binary16 range.  Round-to-nearest-even turns
    |x| >= 65520 into an infinity of the same sign; everything representable stays within the tolerance; the int32
    output is untouched.  Every kernel family (XOR/popcount for wide codes, few tokens, large tiles)."""
    torch, binding = gpu
    case = dict(M=M, N=130, K=2048, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 8200 + M)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    # per-channel scales only, stretched so that the median product sits at the edge of the range
    data["a_scale"] = None
    stretch = 65520.0 / (0.05 * max(1.0, float(np.median(np.abs(want)))))
    data["w_scale"] = (data["w_scale"].astype(np.float32) * np.float32(stretch)).astype(np.float16)
    f = oracle.scale_f64(want, None, data["w_scale"].view(np.uint16))
    over, fin = np.abs(f) >= 65520.0 * (1 + 1e-3), np.abs(f) <= 65504.0
    assert over.sum() > 100 and fin.sum() > 100
    c32, c16 = run_case(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)
    got = c16.astype(np.float64)
    assert np.all(np.isinf(got[over])) and np.array_equal(np.sign(got[over]), np.sign(f[over]))
    assert np.all(np.abs(got[fin] - f[fin]) <= 1e-3 * np.abs(f[fin]) + 1e-6)


@pytest.mark.parametrize("M", [5, 300])
def test_outputs_at_odd_element_offsets(gpu, oracle, M):
    """Outputs that start one element into an allocation: the fp16 output is then 2- but not 4-byte aligned (the tile
    kernels' paired fp16 stores must not be used), the int32 output 4- but not 16-byte aligned."""
    torch, binding = gpu
    dev = torch.device("cuda:0")
    case = dict(M=M, N=256, K=640, p=2, q=1, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 8300 + M)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], 2, 1)
    ap = binding.apmm_pack_activations(torch.from_numpy(data["a_codes"]).to(dev), 2)
    wp = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), 1)
    sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
    raw16 = torch.zeros(M * 256 + 8, dtype=torch.float16, device=dev)
    raw32 = torch.zeros(M * 256 + 8, dtype=torch.int32, device=dev)
    c16, c32 = raw16[1:1 + M * 256].view(M, 256), raw32[1:1 + M * 256].view(M, 256)
    binding.apmm_gemm(M, 256, 640, 2, 1, ap, wp, want_f16=True, w_scale=sw, a_scale=sa, c_i32=c32, c_f16=c16)
    torch.cuda.synchronize()
    assert np.array_equal(c32.cpu().numpy().astype(np.int64), want)
    check_f16(c16.cpu().numpy(), want, data, oracle)
    assert raw16[0].item() == 0 and raw16[1 + M * 256:].abs().sum().item() == 0       # nothing written outside
    assert raw32[0].item() == 0 and raw32[1 + M * 256:].abs().sum().item() == 0


def test_graph_capture_and_replay(gpu, oracle):
    """The calls only enqueue kernels on the given stream, so a serving loop can capture them in a HIP graph:
    pack + GEMM, GEMM from codes and a grouped launch are captured once and replayed several times with other
    work and synchronisations in between; every replay must give the eager (oracle-checked) result."""
    torch, binding = gpu
    dev = torch.device("cuda:0")
    p, q = 2, 2
    case = dict(M=8, N=300, K=1000, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 8200)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    a = torch.from_numpy(data["a_codes"]).to(dev)
    wp = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), q)
    sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
    big = dict(M=300, N=260, K=700, p=p, q=q, a_dist="bernoulli", scaled=False)
    big_data = inputs.make_case(big, 8201)
    big_want = oracle.gemm_i64(big_data["a_codes"], big_data["w_codes"], p, q)
    big_a = torch.from_numpy(big_data["a_codes"]).to(dev)
    big_wp = binding.apmm_pack_weights(torch.from_numpy(big_data["w_codes"]).to(dev), q)
    ap = torch.empty(binding.apmm_packed_activation_bytes(8, 1000, p), dtype=torch.uint8, device=dev)
    big_ap = torch.empty(binding.apmm_packed_activation_bytes(300, 700, p), dtype=torch.uint8, device=dev)
    outs = dict(c1=torch.zeros((8, 300), dtype=torch.int32, device=dev), h1=torch.zeros((8, 300), dtype=torch.float16, device=dev),
                c2=torch.zeros((8, 300), dtype=torch.int32, device=dev), c3=torch.zeros((8, 300), dtype=torch.int32, device=dev),
                c4=torch.zeros((300, 260), dtype=torch.int32, device=dev))

    def work():
        binding.apmm_pack_activations(a, p, out=ap)
        binding.apmm_gemm(8, 300, 1000, p, q, ap, wp, want_f16=True, w_scale=sw, a_scale=sa, c_i32=outs["c1"], c_f16=outs["h1"])
        binding.apmm_gemm_from_codes(a, 300, p, q, wp, c_i32=outs["c2"])
        binding.apmm_gemm_grouped([dict(M=8, N=300, K=1000, a_codes=a, w_packed=wp, c_i32=outs["c3"])], p, q)
        binding.apmm_pack_activations(big_a, p, out=big_ap)
        binding.apmm_gemm(300, 260, 700, p, q, big_ap, big_wp, c_i32=outs["c4"])

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        work()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            work()
    for replay in range(4):
        for t in outs.values():
            t.zero_()                     # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for key in ("c1", "c2", "c3"):
            assert np.array_equal(outs[key].cpu().numpy().astype(np.int64), want), (key, replay)
        check_f16(outs["h1"].cpu().numpy(), want, data, oracle)
        assert np.array_equal(outs["c4"].cpu().numpy().astype(np.int64), big_want), replay


def test_deterministic(gpu):
    case = dict(M=200, N=330, K=1024, p=2, q=2, a_dist="bernoulli", scaled=False)
    data = inputs.make_case(case, 4100)
    first, _ = run_case(gpu, data, case)
    second, _ = run_case(gpu, data, case)
    assert np.array_equal(first, second)


# ----------------------------------------- full-size workload configurations --
def full_check(gpu, oracle, case, seed, also_from_codes=False):
    """Full-size run in the default launch configuration (the one bench.py times); every int32 output and
    every fp16 output is compared with the oracle's (oracle.gemm_i64, oracle.scale_f64)."""
    data = inputs.make_case(case, seed)
    c32, c16 = run_case(gpu, data, case)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], case["p"], case["q"])
    assert c32.shape == want.shape
    assert np.array_equal(c32.astype(np.int64), want)
    if c16 is not None:
        check_f16(c16, want, data, oracle)
    if also_from_codes:
        c32, c16 = run_from_codes(gpu, data, case, workspace=True)
        assert np.array_equal(c32.astype(np.int64), want)
        if data["a_scale"] is not None or data["w_scale"] is not None:
            check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("p,q,M,N,K", [(4, 1, 2000, 2300, 8200), (3, 1, 1100, 4000, 8704), (4, 2, 2000, 2300, 8200),
                                       (4, 2, 500, 5000, 5000), (3, 3, 300, 4200, 2600)])
def test_field_form_tile_arrangements(gpu, oracle, p, q, M, N, K):
    """3- and 4-bit activations at sizes where the launch rule takes each arrangement of the field-form kernels: the
    128 x 256 tile as four wave tiles of 32 x 256 (1-bit weights, K of 8192 or more) and as 2 x 2 wave tiles of
    64 x 128, the 128 x 128 tile as four wave tiles of 32 x 128; ragged borders.  Every int32 and fp16 output
    against the oracle."""
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="normal" if p == 4 else "bernoulli", scaled=True)
    full_check(gpu, oracle, case, 7300 + 10 * p + q + M)


@pytest.mark.parametrize("p,q", [(p, q) for p in range(1, 5) for q in range(1, 5)])
def test_k_split_across_waves_all_widths(gpu, oracle, p, q):
    """The matrix-unit kernel whose four waves split K, asked for by its algo id: several tiles, ragged M, N and K,
    K short enough that some waves get no stage, both outputs."""
    # (the last shape is one round of 64 x 128 tiles but more than 256 of 64 x 64: the wider tile; the others the 64 x 64 one)
    for M, N, K in ((70, 170, 600), (130, 333, 1100 + 512 * q), (64, 160, 100), (300, 3400, 700)):
        case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
        data = inputs.make_case(case, 8100 + 16 * p + q + M)
        want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
        c32, c16 = run_case(gpu, data, case, algo=KSPLIT, want_i32=True, want_f16=True)
        assert np.array_equal(c32.astype(np.int64), want)
        check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("M,N,K,want_i32,want_f16,scaled", [(512, 5120, 10240, False, True, True), (448, 1000, 12800, True, False, False),
                                                            (200, 5001, 10300, True, True, True), (512, 6000, 10240, False, True, True),
                                                            (512, 4096, 4096, True, True, True), (512, 4000, 5120, True, True, True),
                                                            (128, 8192, 1024, False, True, True)])
def test_k_split_across_waves_full_tiles(gpu, oracle, M, N, K, want_i32, want_f16, scaled):
    """Shapes of one round of tiles and long K, where the launch rule itself takes the K-split kernel (the last
    one with 2-bit activations), one output or both, interior and border tiles, an odd output width, each of the four tile
    widths (64 x 64 at 448 x 1001 and 128 x 8192, 64 x 128 at 512 x 4096 / 4000, 64 x 160 at 512 x 5120 and 200 x 5001, 64 x 192 at
    512 x 6000); every output against the oracle."""
    from paper_2409_17870_amd import binding
    p = 2 if N == 4096 else 4
    case = dict(M=M, N=N, K=K, p=p, q=2, a_dist="normal" if p == 4 else "bernoulli", scaled=scaled)
    data = inputs.make_case(case, 8200 + M)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, 2)
    c32, c16 = run_case(gpu, data, case, want_i32=want_i32, want_f16=want_f16)
    assert binding.apmm_last_gemm_kernel().startswith("gemm_mfma_ksplit_kernel")
    if want_i32:
        assert np.array_equal(c32.astype(np.int64), want)
    if want_f16:
        check_f16(c16, want, data, oracle)


def test_k_split_kernel_declines_wide_codes(gpu):
    torch, binding = gpu
    a = torch.zeros((64, 512), dtype=torch.uint8, device="cuda:0")
    w = torch.zeros((64, 512), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(binding.ApmmError):
        binding.apmm_gemm(64, 64, 512, 5, 2, binding.apmm_pack_activations(a, 5), binding.apmm_pack_weights(w, 2), algo=KSPLIT)


@pytest.mark.parametrize("M,N,K,p,q", [(65, 4096, 700, 2, 2), (128, 1000, 512, 1, 1), (300, 4000, 3100, 2, 1), (512, 4096, 3072, 1, 2)])
def test_k_split_rule_for_group_form_activations(gpu, oracle, M, N, K, p, q):
    """1- and 2-bit activations on outputs of one round of 64 x 128 tiles: the launch rule takes the K-split kernel up
    to 128 tokens at any K and from K = 3072 on; int32 and fp16 outputs against the oracle."""
    from paper_2409_17870_amd import binding
    case = dict(M=M, N=N, K=K, p=p, q=q, a_dist="bernoulli", scaled=True)
    data = inputs.make_case(case, 8300 + M)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    c32, c16 = run_case(gpu, data, case, want_i32=True, want_f16=True)
    assert binding.apmm_last_gemm_kernel().startswith("gemm_mfma_ksplit_kernel")
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


def test_config2_square_4096_w1a2(gpu, oracle):
    full_check(gpu, oracle, inputs.config_cases(2)[0], inputs.BASE_SEED + 2)


@pytest.mark.parametrize("idx", range(9))
def test_config3_decode_w2a2(gpu, oracle, idx):
    """Decode shapes, whole outputs against the oracle, through both ways the activations can arrive: packed by
    apmm_pack_activations (then apmm_gemm) and as codes (apmm_gemm_from_codes, the one-launch form these shapes
    take and the one the decode timings are quoted on)."""
    case = inputs.config_cases(3)[idx]
    data = inputs.make_case(case, inputs.BASE_SEED + 3)
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], case["p"], case["q"])
    c32, c16 = run_case(gpu, data, case, want_i32=True, want_f16=True)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)
    c32, c16 = run_from_codes(gpu, data, case)
    assert np.array_equal(c32.astype(np.int64), want)
    check_f16(c16, want, data, oracle)


@pytest.mark.parametrize("idx", range(6))
def test_config4_prefill_w1a4_w2a4(gpu, oracle, idx):
    full_check(gpu, oracle, inputs.config_cases(4)[idx], inputs.BASE_SEED + 4)


@pytest.mark.parametrize("idx", range(7))
def test_config5_decoder_layer_w2a4(gpu, oracle, idx):
    """All seven linears of the layer (q, k, v, o, gate, up, down), each with its own seeded inputs, through
    apmm_pack_activations + apmm_gemm and through apmm_gemm_from_codes with a workspace (online packing)."""
    case = inputs.config_cases(5)[idx]
    full_check(gpu, oracle, case, inputs.BASE_SEED + 5 + idx, also_from_codes=True)
