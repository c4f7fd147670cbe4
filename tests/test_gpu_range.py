"""Range of the d = 64 kernels that form fp32 products from bf16 pieces on the matrix cores (needs the GPU).

num and den are homogeneous in Q, K, V and Phi_hat under the identity and ReLU maps, and scaling by a power of two is
exact in fp32.  A kernel whose products are fp32-grade must therefore return bit-identical mantissas when the inputs
are scaled by powers of two, as long as no piece of any operand leaves the range of bf16: the third piece of x holds
bits down to 2^-23 |x| and bf16 reaches down to 2^-133 (its subnormals are honoured), so the scaling is exact for
operands of magnitude 2^-110 and more and degrades gradually below; at the top, a bf16 number has the range of an fp32
number.  Covers both forms of the fused forward pass (short lists several buckets per wavefront, long lists through
S_l)."""
import numpy as np
import pytest

from paper_2410_03462_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grf():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_03462_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def problem():
    rng = np.random.default_rng(0)
    n, rp, col, val = synth.columns_of_lengths(list(rng.integers(0, 60, size=200)), rng)      # lists on both sides of 17 and 32
    Q, K, V = synth.qkv(1, 2, n, 64, np.random.default_rng(1))
    # keep every element at 2^-12 or more in magnitude, so that the exact range below is a statement about the scales
    for x in (Q, K, V):
        small = np.abs(x) < 2.0 ** -12
        x[small] = np.where(x[small] < 0, -(2.0 ** -12), 2.0 ** -12)
    return n, rp, col, val, Q, K, V


def run(grf, problem, a, b, c, e, feature_map):
    import torch
    n, rp, col, val, Q, K, V = problem
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x.astype(np.float32))).cuda()
    two = np.float32(2.0)
    phi = grf.Phi.from_host(n, rp, col, val * two ** e)
    _, num, den = grf.grf_masked_linear_attention_fused(dev(Q * two ** a), dev(K * two ** b), dev(V * two ** c), phi, feature_map,
                                                        return_num_den=True)
    return num.cpu().numpy().astype(np.float64), den.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("feature_map", ["identity", "relu"])
@pytest.mark.parametrize("scales", [(40, -40, 0, 0), (-40, 40, 20, -10), (0, 0, 100, 0), (0, 0, -90, 0), (95, -95, 0, 0), (-95, 95, 0, 0),
                                    (0, 0, 0, 30), (0, 0, 0, -30), (30, 30, 30, 0), (-30, -30, -30, 0), (0, -95, 95, 0)])
def test_scaling_by_powers_of_two_is_exact(grf, problem, scales, feature_map):
    """Scales 2^a, 2^b, 2^c, 2^e on Q, K, V, Phi_hat with every operand at 2^-107 or more and every result in range."""
    a, b, c, e = scales
    num0, den0 = run(grf, problem, 0, 0, 0, 0, feature_map)
    num, den = run(grf, problem, a, b, c, e, feature_map)
    assert np.array_equal(num, num0 * 2.0 ** (a + b + c + 2 * e))
    assert np.array_equal(den, den0 * 2.0 ** (a + b + 2 * e))


@pytest.mark.parametrize("scale,bar", [(-100, 1e-6), (-110, 1e-5), (-120, 1e-3)])
def test_small_end_degrades_gradually(grf, problem, scale, bar):
    """Below 2^-110 an operand's low pieces fall under the smallest bf16 subnormal: with V at 2^-12 .. 4 times the scale,
    the error stays far below the fp32 bar at 2^-100, reaches it near 2^-110 and is still small at 2^-120."""
    num0, den0 = run(grf, problem, 0, 0, 0, 0, "relu")
    num, den = run(grf, problem, 0, 0, scale, 0, "relu")
    assert np.array_equal(den, den0)
    assert np.abs(num / 2.0 ** scale - num0).max() <= bar * np.abs(num0).max()
