"""Short column lists at d = 64 (needs the GPU): lists of at most 17 entries are evaluated several buckets per
wavefront, in windows of the entry sequence that hold whole buckets; longer lists one bucket per wavefront.  Hand-made
feature matrices put lists of every short length side by side, at the window and tile boundaries, and next to long
ones; the bucket-fused forward pass and the backward pass are compared with the CPU checker."""
import numpy as np
import pytest

from paper_2410_03462_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
FEATURE_MAP_CODE = {"relu": 0, "identity": 1, "elu1": 2}


@pytest.fixture(scope="module")
def grf():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2410_03462_amd import binding
    binding.lib()
    return binding


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    return float(np.abs(x - ref).max() / scale) if scale > 0 else float(np.abs(x).max())


def to_dev(x, dtype="f32"):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def length_patterns():
    rng = np.random.default_rng(17)
    up = list(range(1, 18))
    yield "1_to_17_and_back", up + up[::-1] + [4] * 20
    yield "all_ones", [1] * 100
    yield "all_16", [16] * 40
    yield "all_17", [17] * 40
    yield "17_and_18_alternating", [17, 18] * 20
    yield "short_between_long", [3, 40, 5, 18, 17, 17, 17, 1, 100, 2, 0, 0, 9, 33, 1, 1, 1, 64, 16, 16, 15, 129] + [2] * 110
    yield "empty_columns_around", [0, 0, 5, 0, 0, 0, 0, 12, 0, 17, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 7, 0, 0] + [3] * 20
    yield "window_edges", [15, 1, 16, 16, 1, 15, 17, 14, 2, 1, 13, 17, 17, 15, 17, 1, 1, 14, 16, 17, 3] + [5] * 30
    yield "random_0_17", list(rng.integers(0, 18, size=300))
    yield "random_0_40", list(rng.integers(0, 41, size=300))
    yield "mostly_seven", list(np.clip(rng.poisson(7, size=400), 0, 30))


PATTERNS = dict(length_patterns())


@pytest.mark.parametrize("name", list(PATTERNS))
@pytest.mark.parametrize("dtype,feature_map", [("f32", "relu"), ("bf16", "relu"), ("f32", "elu1"), ("bf16", "elu1")])
def test_fused_forward_short_lists(grf, oracle, name, dtype, feature_map):
    rng = np.random.default_rng([len(name), 1])
    n, rp, col, val = synth.columns_of_lengths(PATTERNS[name], rng)
    assert np.array_equal(np.bincount(col, minlength=n), np.asarray(PATTERNS[name]))
    Q, K, V = synth.qkv(2, 2, n, 64, np.random.default_rng([len(name), 2]), dtype)
    fm = FEATURE_MAP_CODE[feature_map]
    ref = oracle.masked_linear_attention(Q, K, V, rp, col, val, feature_map=fm)
    # the same sums with every term replaced by its magnitude (phi >= 0 for both maps): the scale of each element's rounding
    mag = oracle.masked_linear_attention(Q, K, np.abs(V), rp, col, np.abs(val), feature_map=fm)
    phi = grf.Phi.from_host(n, rp, col, val)
    out, num, den = grf.grf_masked_linear_attention_fused(*(to_dev(x, dtype) for x in (Q, K, V)), phi, feature_map, return_num_den=True)
    num, den = num.cpu().numpy(), den.cpu().numpy()
    tol = TOL[dtype]
    assert relerr(num, ref["num"]) <= tol and relerr(den, ref["den"]) <= tol
    # element by element: relative to the element itself plus a few units of rounding of its terms' magnitudes
    floor = 2.0 ** -20 if dtype == "f32" else 2.0 ** -13
    assert np.all(np.abs(num - ref["num"]) <= tol * np.abs(ref["num"]) + floor * mag["num"])
    assert np.all(np.abs(den - ref["den"]) <= tol * np.abs(ref["den"]) + floor * mag["den"])
    # rows without entries: num = den = 0
    empty = np.diff(rp) == 0
    assert np.all(num[:, :, empty] == 0) and np.all(den[:, :, empty] == 0)
    # bitwise reproducible, also when the slices go through in chunks
    _, num2, den2 = grf.grf_masked_linear_attention_fused(*(to_dev(x, dtype) for x in (Q, K, V)), phi, feature_map, bh_chunk=3, return_num_den=True)
    assert np.array_equal(num, num2.cpu().numpy()) and np.array_equal(den, den2.cpu().numpy())


@pytest.mark.parametrize("name", list(PATTERNS))
@pytest.mark.parametrize("dtype,feature_map", [("f32", "relu"), ("bf16", "elu1")])
def test_backward_short_lists(grf, oracle, name, dtype, feature_map):
    rng = np.random.default_rng([len(name), 3])
    n, rp, col, val = synth.columns_of_lengths(PATTERNS[name], rng)
    if (np.diff(rp) == 0).any():
        pytest.skip("a row without entries has den = 0: no gradient to compare")
    if max(PATTERNS[name]) == 1:
        pytest.skip("one entry per list: every row attends to one key, out_i = v_j, and all gradients but dV cancel to zero exactly")
    Q, K, V = synth.qkv(1, 2, n, 64, np.random.default_rng([len(name), 4]), dtype)
    fm = FEATURE_MAP_CODE[feature_map]
    fwd = oracle.masked_linear_attention(Q, K, V, rp, col, val, feature_map=fm)
    out32, den32 = fwd["out"].astype(np.float32), fwd["den"].astype(np.float32)
    assert np.isfinite(out32).all() and (den32 > 0).all()
    d_out = np.random.default_rng([len(name), 5]).standard_normal(Q.shape).astype(np.float32)
    ref = oracle.masked_linear_attention_backward(Q, K, V, rp, col, val, out32, den32, d_out, fm)
    phi = grf.Phi.from_host(n, rp, col, val)
    got = grf.grf_masked_linear_attention_backward(*(to_dev(x, dtype) for x in (Q, K, V)), phi, to_dev(out32), to_dev(den32),
                                                   to_dev(d_out), feature_map)
    host = [t.cpu().numpy() for t in got]
    host[3] = host[3][:, : phi.nnz]
    for label, x, r in zip(("dQ", "dK", "dV", "dphi"), host, ref):
        assert np.isfinite(x).all(), label
        assert relerr(x, r) <= TOL[dtype], (label, relerr(x, r))


@pytest.mark.parametrize("name", ["1_to_17_and_back", "short_between_long", "window_edges", "random_0_40"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_short_lists_with_one_value_plane_per_head(grf, oracle, name, dtype):
    """Per-head modulation (Sec. 4): the heads share the pattern, each has its own values, and the planes' stride is the
    capacity of Phi_hat's buffers, here larger than nnz.  Forward and backward against the CPU checker, head by head."""
    import torch
    rng = np.random.default_rng([len(name), 6])
    n, rp, col, val = synth.columns_of_lengths(PATTERNS[name], rng)
    if (np.diff(rp) == 0).any():
        pytest.skip("a row without entries has den = 0: no gradient to compare")
    H = 3
    val = np.ravel(val)
    vals = np.stack([val * rng.uniform(0.5, 1.5, size=val.shape).astype(np.float32) for _ in range(H)])
    Q, K, V = synth.qkv(2, H, n, 64, np.random.default_rng([len(name), 7]), dtype)
    ref = oracle.masked_linear_attention(Q, K, V, rp, col, vals)
    nnz, cap = col.shape[0], col.shape[0] + 37
    col_pad = np.concatenate([col, np.full(37, -1, np.int32)])
    vals_pad = np.concatenate([vals, np.full((H, 37), np.nan, np.float32)], axis=1)
    phi = grf.Phi.from_host(n, rp, col_pad, vals_pad)
    phi.nnz = nnz
    assert phi.capacity == cap
    dev = [to_dev(x, dtype) for x in (Q, K, V)]
    out, num, den = grf.grf_masked_linear_attention_fused(*dev, phi, "relu", return_num_den=True)
    tol = TOL[dtype]
    assert relerr(num.cpu().numpy(), ref["num"]) <= tol and relerr(den.cpu().numpy(), ref["den"]) <= tol
    out32, den32 = ref["out"].astype(np.float32), ref["den"].astype(np.float32)
    assert np.isfinite(out32).all() and (den32 > 0).all()
    d_out = np.random.default_rng([len(name), 8]).standard_normal(Q.shape).astype(np.float32)
    gref = oracle.masked_linear_attention_backward(Q, K, V, rp, col, vals, out32, den32, d_out, 0)
    got = grf.grf_masked_linear_attention_backward(*dev, phi, to_dev(out32), to_dev(den32), to_dev(d_out), "relu")
    host = [t.cpu().numpy() for t in got]
    assert host[3].shape[0] == H
    host[3] = host[3][:, :nnz]
    for label, x, r in zip(("dQ", "dK", "dV", "dphi"), host, gref):
        assert np.isfinite(x).all(), label
        assert relerr(x, r) <= tol, (label, relerr(x, r))
