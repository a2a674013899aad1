"""Seeded synthetic inputs for the bipolar-INT GEMM workloads.

This module produces *data* only: code matrices (one uint8 per element) and
binary16 scale vectors.  It holds none of the method's arithmetic, so both
the CPU oracle's tests and the GPU path can be fed from it.  Everything is a
pure function of (seed, tag, element index) through a counter-based
splitmix64 hash, so any element can be regenerated on its own.

The shapes stand in for the paper's workloads: the square MatMuls of Table 1
and the Llama-2-7B linear shapes of Table 2 (the paper fixes only shapes;
integer GEMM time does not depend on the values).  The paper's models and
quantised weights are not available, so codes are drawn at random:
Bernoulli(1/2) bits, or a discretised normal for 4-bit activations.
"""
import numpy as np

TAG_A, TAG_W, TAG_W_SCALE, TAG_A_SCALE = 1, 2, 3, 4
BASE_SEED = 20240917

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(x):
    """Finaliser of the splitmix64 generator applied to a uint64 array of counters."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _hash(seed, tag, count, offset=0):
    idx = np.arange(offset, offset + count, dtype=np.uint64)
    key = np.uint64(seed) ^ (np.uint64(tag) << np.uint64(56))
    return splitmix64(key ^ idx)


def bernoulli_codes(seed, tag, rows, K, bits):
    """rows x K codes whose `bits` bits are i.i.d. Bernoulli(1/2)."""
    h = _hash(seed, tag, rows * K)
    return (h >> np.uint64(64 - bits)).astype(np.uint8).reshape(rows, K)


def uniform01(seed, tag, count):
    h = _hash(seed, tag, count)
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def normal_codes(seed, tag, rows, K, bits=4, sigma_steps=5.0):
    """Codes from a discretised N(0,1) clipped to the code range.

    z ~ N(0,1) by Box-Muller on two hashed uniforms; t = sigma_steps*z is binned
    into cells of width 2 centred on the odd integers, and the bin index is
    clipped to [0, 2^bits - 1].  With bits=4 and sigma_steps=5, three sigma
    lands on the outermost code.
    """
    n = rows * K
    u1 = uniform01(seed, tag, n)
    u2 = uniform01(seed ^ 0x5DEECE66D, tag, n)
    z = np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)
    cell = np.floor(sigma_steps * z / 2.0).astype(np.int64) + (1 << (bits - 1))
    return np.clip(cell, 0, (1 << bits) - 1).astype(np.uint8).reshape(rows, K)


def normal_features_f16(seed, tag, rows, K, outlier_every=0):
    """rows x K binary16 features ~ N(0,1) (Box-Muller on hashed uniforms); with outlier_every > 0 every
    outlier_every-th column is multiplied by 8, the heavy-tailed channels that activations of language
    models show.  Input of the fused quantise + pack step."""
    n = rows * K
    u1 = uniform01(seed, tag, n)
    u2 = uniform01(seed ^ 0x5DEECE66D, tag, n)
    z = (np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)).reshape(rows, K)
    if outlier_every:
        z[:, ::outlier_every] *= 8.0
    return z.astype(np.float16)


def scales_f16(seed, tag, count, lo=0.01, hi=0.1):
    """binary16 scale vector ~ U(lo, hi); returned as float16 (view as uint16 for bit patterns)."""
    u = uniform01(seed, tag, count)
    return (lo + (hi - lo) * u).astype(np.float16)


# ----------------------------------------------------------------------------
# The five workload configurations (index = seed offset).
# ----------------------------------------------------------------------------
LLAMA7B_NK = [(4096, 4096), (11008, 4096), (4096, 11008)]
DECODER13B_NK = [(5120, 5120)] * 4 + [(13824, 5120)] * 2 + [(5120, 13824)]


def config_cases(index):
    """List of dicts {M,N,K,p,q,a_dist,scaled} for workload configuration `index` (1..5)."""
    if index == 1:
        return [dict(M=16, N=256, K=512, p=2, q=1, a_dist="bernoulli", scaled=False)]
    if index == 2:
        return [dict(M=4096, N=4096, K=4096, p=2, q=1, a_dist="bernoulli", scaled=False)]
    if index == 3:
        return [dict(M=M, N=N, K=K, p=2, q=2, a_dist="bernoulli", scaled=True)
                for M in (1, 8, 16) for (N, K) in LLAMA7B_NK]
    if index == 4:
        return [dict(M=2048, N=N, K=K, p=4, q=q, a_dist="normal", scaled=True)
                for q in (1, 2) for (N, K) in LLAMA7B_NK]
    if index == 5:
        return [dict(M=512, N=N, K=K, p=4, q=2, a_dist="bernoulli", scaled=True)
                for (N, K) in DECODER13B_NK]
    raise ValueError("configuration index must be 1..5")


def make_case(case, seed):
    """Materialise one case: returns dict with a_codes, w_codes, a_scale, w_scale (float16 or None)."""
    M, N, K, p, q = case["M"], case["N"], case["K"], case["p"], case["q"]
    if case.get("a_dist", "bernoulli") == "normal":
        a = normal_codes(seed, TAG_A, M, K, bits=p)
    else:
        a = bernoulli_codes(seed, TAG_A, M, K, p)
    w = bernoulli_codes(seed, TAG_W, N, K, q)
    out = dict(a_codes=a, w_codes=w, a_scale=None, w_scale=None)
    if case.get("scaled", False):
        out["w_scale"] = scales_f16(seed, TAG_W_SCALE, N)
        out["a_scale"] = scales_f16(seed, TAG_A_SCALE, M)
    return out
