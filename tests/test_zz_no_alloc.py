"""The entry point that allocates nothing (apmm_gemm_from_codes_noalloc): its packed activations live in a
buffer inside the library's device code.  Checked through the C ABI against apmm_gemm_from_codes with a
caller-supplied workspace (the existing entry point it is a variant of) and against the oracle, on two calls in
a row, the second with a smaller input, so that what the first call left in the shared buffer would show."""
import numpy as np
import pytest

from paper_2409_17870_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2409_17870_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return torch, binding


def _both_ways(gpu, oracle, case, seed):
    torch, binding = gpu
    dev = torch.device("cuda:0")
    M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
    data = inputs.make_case(case, seed)
    a = torch.from_numpy(data["a_codes"]).to(dev)
    wp = binding.apmm_pack_weights(torch.from_numpy(data["w_codes"]).to(dev), q)
    sa, sw = torch.from_numpy(data["a_scale"]).to(dev), torch.from_numpy(data["w_scale"]).to(dev)
    # the existing entry point, with a workspace of the caller's
    ws = torch.empty(binding.apmm_packed_activation_bytes(M, K, p), dtype=torch.uint8, device=dev)
    ref32, ref16 = binding.apmm_gemm_from_codes(a, N, p, q, wp, want_i32=True, want_f16=True, w_scale=sw, a_scale=sa,
                                                workspace=ws)
    # the entry point under test: outputs preallocated, nothing allocated during the call
    c32 = torch.full((M, N), -7, dtype=torch.int32, device=dev)
    c16 = torch.full((M, N), -7, dtype=torch.float16, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.apmm_gemm_from_codes_noalloc(a, N, p, q, wp, c_i32=c32, c_f16=c16, w_scale=sw, a_scale=sa)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(c32, ref32)
    assert torch.equal(c16.view(torch.int16), ref16.view(torch.int16))
    want = oracle.gemm_i64(data["a_codes"], data["w_codes"], p, q)
    assert np.array_equal(c32.cpu().numpy().astype(np.int64), want)
    f = oracle.scale_f64(want, data["a_scale"].view(np.uint16), data["w_scale"].view(np.uint16))
    got = c16.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - f) <= 1e-3 * np.abs(f) + 1e-6)


def test_noalloc_two_calls_second_smaller(gpu, oracle):
    """Shapes that go through the packed buffer (too many tokens for the one-launch kernels): group form (2-bit)
    and field form (4-bit) activations, ragged M, N, K; the second call of each pair is smaller in M and K."""
    _both_ways(gpu, oracle, dict(M=300, N=260, K=1100, p=2, q=2, a_dist="bernoulli", scaled=True), 9901)
    _both_ways(gpu, oracle, dict(M=70, N=130, K=500, p=2, q=2, a_dist="bernoulli", scaled=True), 9902)
    _both_ways(gpu, oracle, dict(M=257, N=200, K=1500, p=4, q=2, a_dist="normal", scaled=True), 9903)
    _both_ways(gpu, oracle, dict(M=100, N=96, K=640, p=4, q=1, a_dist="normal", scaled=True), 9904)
    # few tokens: the one-launch kernels serve the call, the buffer is not touched
    _both_ways(gpu, oracle, dict(M=5, N=203, K=1100, p=2, q=2, a_dist="bernoulli", scaled=True), 9905)


def test_noalloc_rejects_what_does_not_fit(gpu):
    torch, binding = gpu
    dev = torch.device("cuda:0")
    M, K, p, q = 4096, 8192 + 512, 2, 1          # 4096 x 8704 x 2 bits > 8 MiB
    assert binding.apmm_packed_activation_bytes(M, K, p) > binding.NOALLOC_MAX_PACKED_BYTES
    a = torch.zeros((M, K), dtype=torch.uint8, device=dev)
    wp = binding.apmm_pack_weights(torch.zeros((32, K), dtype=torch.uint8, device=dev), q)
    c32 = torch.full((M, 32), -7, dtype=torch.int32, device=dev)
    with pytest.raises(binding.ApmmError) as err:
        binding.apmm_gemm_from_codes_noalloc(a, 32, p, q, wp, c_i32=c32)
    assert err.value.status == 4 and "8388608" in str(err.value)
    torch.cuda.synchronize()
    assert int((c32 != -7).sum().item()) == 0     # nothing was launched
