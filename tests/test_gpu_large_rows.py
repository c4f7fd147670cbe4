"""Rows of Phi_hat with many possible deposits (needs the GPU): beyond 768 possible deposits per node a workgroup per
node can order the deposits with a sorting network instead of one wavefront ranking them by counting; up to 8192 both
kernels can serve and the library picks one by a cost model, beyond that only the workgroup kernel.  Every test runs
four times: with the library's choice, with either kernel forced wherever both can serve, and with the wavefront kernel
ordering by (column, slot) as two words (the form it takes when they do not fit one 32-bit key).  Pattern bit-exact, values
within 1e-5, against the CPU checker, on both sides of the limits, at the largest supported size, with more nodes than
workgroups, and through the gradient with respect to f."""
import numpy as np
import pytest

from paper_2410_03462_amd import synth

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5


@pytest.fixture(scope="module")
def grf():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_03462_amd import binding
    binding.lib()
    return binding


@pytest.fixture(autouse=True, params=["chosen", "wavefront", "workgroup", "wavefront_two_word_keys"])
def row_kernel(request, grf):
    grf.grf_debug_force_row_kernel({"chosen": 0, "wavefront": 1, "workgroup": 2, "wavefront_two_word_keys": 3}[request.param])
    yield request.param
    grf.grf_debug_force_row_kernel(0)


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    return float(np.abs(x - ref).max() / scale) if scale > 0 else float(np.abs(x).max())


def check_sample(grf, oracle, g_host, f, p_halt, n_walks, seed):
    g = grf.DeviceGraph.from_host(g_host)
    phi = grf.grf_sample(g, f, p_halt, n_walks, seed)
    rp, col, val = phi.to_host()
    rp0, col0, val0 = oracle.sample(g_host, f, p_halt, n_walks, seed)
    assert np.array_equal(rp, rp0) and np.array_equal(col, col0)
    for h in range(f.shape[0]):
        assert relerr(val[h], val0[h]) <= TOL_F32, (h, relerr(val[h], val0[h]))
        # element by element: a few units of rounding of the deposits' magnitudes (the checker run on |f| with the
        # same walks gives the sum of magnitudes of every entry, the loads being positive)
    _, _, mag = oracle.sample(g_host, np.abs(f), p_halt, n_walks, seed)
    assert np.all(np.abs(val - val0) <= TOL_F32 * np.abs(val0) + 2.0 ** -20 * mag)
    # a second run gives the same bits
    rp2, col2, val2 = grf.grf_sample(g, f, p_halt, n_walks, seed).to_host()
    assert np.array_equal(rp2, rp) and np.array_equal(col2, col) and np.array_equal(val2, val)
    return phi, (rp0, col0, val0)


def test_image_setting_of_the_paper(grf, oracle):
    """App. C, hyperparameter table (ImageNet): 100 walks per node, i_max = 100, p_halt = 0.1, on a 14 x 14 grid of
    patches: up to 10 001 deposits per node."""
    g_host = synth.grid_graph(14, 14, 4)
    f = synth.modulation(101, np.random.default_rng(14), n_f=2)
    check_sample(grf, oracle, g_host, f, 0.1, 100, 7)


@pytest.mark.parametrize("n_walks,f_len", [(13, 60), (12, 65), (48, 65), (90, 92), (8191, 2), (64, 129), (127, 130)])
def test_rows_filled_to_the_bound(grf, oracle, n_walks, f_len):
    """No halting, so every row holds exactly 1 + n_walks (f_len - 1) deposits: 768 and 769 (either side of the switch
    between the two kernels), 3073, 8191, 8192 (more walks than the workgroup has threads), 8193, and 16384 (the most)."""
    g_host = synth.grid_graph(5, 4, 8)
    f = synth.modulation(f_len, np.random.default_rng(f_len))
    check_sample(grf, oracle, g_host, f, 0.0, n_walks, 3 * n_walks)


def test_more_nodes_than_workgroups_isolated_nodes_and_halting(grf, oracle):
    rng = np.random.default_rng(8)
    g_host = synth.random_graph(1300, 5.0, rng, weights="sym_norm", isolated=7)
    f = synth.modulation(65, rng, n_f=3)
    check_sample(grf, oracle, g_host, f, 0.3, 48, 99)
    # p_halt = 1: every row is its diagonal entry f_0
    g = grf.DeviceGraph.from_host(g_host)
    rp, col, val = grf.grf_sample(g, f, 1.0, 48, 1).to_host()
    assert np.array_equal(rp, np.arange(1301)) and np.array_equal(col, np.arange(1300))
    assert relerr(val, np.repeat(f[:, :1], 1300, axis=1)) <= 2e-7


def test_one_deposit_more_than_supported_is_refused(grf):
    g = grf.DeviceGraph.from_host(synth.grid_graph(5, 4, 8))
    with pytest.raises(grf.GrfError) as e:
        grf.grf_sample(g, np.ones((1, 129), np.float32), 0.5, 128, 0)      # 1 + 128 * 128 = 16385
    assert e.value.status == grf.GRF_EUNSUPPORTED


@pytest.mark.parametrize("n_walks,f_len,p_halt", [(100, 101, 0.1), (48, 65, 0.0), (2000, 4, 0.2)])
def test_gradient_with_respect_to_f(grf, oracle, n_walks, f_len, p_halt):
    """grf_sample_backward over rows assembled by workgroups, fed with a synthetic dPhi_hat, against the checker."""
    import torch
    g_host = synth.grid_graph(9, 7, 8)
    f = synth.modulation(f_len, np.random.default_rng(5), n_f=2)
    phi, (rp0, col0, val0) = check_sample(grf, oracle, g_host, f, p_halt, n_walks, 21)
    dphi = np.random.default_rng(6).standard_normal((2, phi.capacity)).astype(np.float32)
    g = grf.DeviceGraph.from_host(g_host)
    df = grf.grf_sample_backward(g, f_len, p_halt, n_walks, 21, phi, torch.from_numpy(dphi).cuda()).cpu().numpy()
    want = oracle.sample_backward(g_host, f_len, p_halt, n_walks, 21, rp0, col0, dphi[:, : phi.nnz])
    # per hop count: against the sum of the magnitudes of its terms (the loads are positive)
    mag = oracle.sample_backward(g_host, f_len, p_halt, n_walks, 21, rp0, col0, np.abs(dphi[:, : phi.nnz]))
    assert np.all(np.abs(df - want) <= TOL_F32 * np.abs(want) + 2.0 ** -20 * mag)
    df2 = grf.grf_sample_backward(g, f_len, p_halt, n_walks, 21, phi, torch.from_numpy(dphi).cuda()).cpu().numpy()
    assert np.array_equal(df, df2)


@pytest.mark.parametrize("n_walks,f_len,p_halt", [(64, 16, 0.2), (100, 51, 0.1), (64, 33, 0.0)])
def test_both_kernels_give_the_same_pattern(grf, n_walks, f_len, p_halt, row_kernel):
    """Where both kernels can serve (769 .. 8192 possible deposits): row_ptr and col are the same bits, the values differ
    by the order of their sums only; the library's own choice is one of the two, bit for bit."""
    if row_kernel != "chosen":
        pytest.skip("forces the kernels itself")
    rng = np.random.default_rng(n_walks)
    g_host = synth.knn_graph(rng.random((700, 3)), 6, "exp")
    g = grf.DeviceGraph.from_host(g_host)
    f = synth.modulation(f_len, rng, n_f=2)
    got = {}
    for which in (0, 1, 2, 3):
        grf.grf_debug_force_row_kernel(which)
        got[which] = grf.grf_sample(g, f, p_halt, n_walks, 11).to_host()
    grf.grf_debug_force_row_kernel(0)
    assert np.array_equal(got[1][0], got[2][0]) and np.array_equal(got[1][1], got[2][1])
    assert relerr(got[1][2], got[2][2]) <= 2e-6
    assert all(np.array_equal(a, b) for a, b in zip(got[1], got[3]))      # one key or two words: the same order, the same bits
    assert any(all(np.array_equal(a, b) for a, b in zip(got[0], got[k])) for k in (1, 2))
