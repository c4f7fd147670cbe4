"""Prepared column lists (needs the GPU): grf_phi_prepare once, then the *_prepared attention calls must return the
bits of the calls that rebuild the lists; grf_phi_prepare_values follows a changed modulation f over the same walks."""
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


def to_dev(x, dtype="f32"):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def same(a, b):
    import torch
    return torch.equal(torch.nan_to_num(a, nan=7.0, posinf=8.0, neginf=9.0), torch.nan_to_num(b, nan=7.0, posinf=8.0, neginf=9.0))


def workloads():
    rng = np.random.default_rng(31)
    yield "tiny_grid_d32", synth.workload("tiny_grid")
    wl = synth.workload("vit_grid"); wl.B, wl.H = 2, 3
    yield "vit_grid_b2h3", wl
    g = synth.random_graph(777, 6.0, rng, weights="sym_norm", isolated=5)
    yield "random_777", synth.Workload("random_777", g, synth.modulation(9, rng), 0.3, 11, 2, 2, 64, "f32")
    g = synth.knn_graph(synth.uniform_points(3000, rng), 12, "gauss")      # lists on both sides of 17 and 32 entries
    yield "cloud_3k_perhead_bf16", synth.Workload("cloud_3k", g, synth.modulation(12, rng, n_f=3), 0.25, 16, 2, 3, 64, "bf16")


WORKLOADS = dict(workloads())


@pytest.mark.parametrize("name", list(WORKLOADS))
def test_prepared_calls_give_the_bits_of_the_rebuilding_calls(grf, name):
    import torch
    wl = WORKLOADS[name]
    g = grf.DeviceGraph.from_host(wl.graph)
    phi = grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    Q, K, V = (to_dev(x, wl.dtype) for x in wl.qkv())
    prepared = grf.grf_phi_prepare(phi)
    assert prepared.numel() >= grf.grf_phi_prepare_bytes(phi.n, phi.nnz, phi.n_f)

    assert same(grf.grf_form_buckets(K, V, phi), grf.grf_form_buckets_prepared(K, V, phi, prepared))
    for chunk in (0, 2):
        want = grf.grf_masked_linear_attention(Q, K, V, phi, bh_chunk=chunk, return_num_den=True)
        got = grf.grf_masked_linear_attention_prepared(Q, K, V, phi, prepared, bh_chunk=chunk, return_num_den=True)
        assert all(same(a, b) for a, b in zip(got, want))
        want = grf.grf_masked_linear_attention_fused(Q, K, V, phi, bh_chunk=chunk, return_num_den=True)
        got = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, prepared, bh_chunk=chunk, return_num_den=True)
        assert all(same(a, b) for a, b in zip(got, want))
    out, _, den = want
    d_out = torch.randn(out.shape, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    ok = torch.isfinite(out).all(dim=-1) & (den != 0)
    out = torch.where(ok[..., None], out, torch.ones_like(out)); den = torch.where(ok, den, torch.ones_like(den))
    want = grf.grf_masked_linear_attention_backward(Q, K, V, phi, out, den, d_out)
    got = grf.grf_masked_linear_attention_backward_prepared(Q, K, V, phi, prepared, out, den, d_out)
    for a, b in zip(got, want):
        assert same(a[..., : phi.nnz] if a.shape == (phi.n_f, phi.capacity) else a, b[..., : phi.nnz] if b.shape == (phi.n_f, phi.capacity) else b)
    # the buffer is only read: a second round gives the same bits
    again = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, prepared, return_num_den=True)
    assert all(same(a, b) for a, b in zip(again, grf.grf_masked_linear_attention_fused(Q, K, V, phi, return_num_den=True)))


def test_values_refresh_follows_a_new_modulation(grf):
    rng = np.random.default_rng(32)
    wl = WORKLOADS["random_777"]
    g = grf.DeviceGraph.from_host(wl.graph)
    phi = grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    Q, K, V = (to_dev(x) for x in wl.qkv())
    prepared = grf.grf_phi_prepare(phi)
    before = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, prepared, return_num_den=True)
    # a new f over the same walks: the pattern stays, the values change
    f2 = synth.modulation(wl.f_len, rng)
    col_before = phi.col.clone()
    grf.grf_sample(g, f2, wl.p_halt, wl.n_walks, wl.walk_seed, out=phi)
    assert same(phi.col, col_before)
    want = grf.grf_masked_linear_attention_fused(Q, K, V, phi, return_num_den=True)
    stale = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, prepared, return_num_den=True)
    assert not same(stale[1], want[1])      # the buckets would still be formed from the old values in list order
    grf.grf_phi_prepare_values(phi, prepared)
    fresh = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, prepared, return_num_den=True)
    assert all(same(a, b) for a, b in zip(fresh, want))
    assert not same(fresh[1], before[1])


def test_prepared_with_the_entry_count_left_on_the_device(grf):
    """Phi_hat sampled without a host round trip (nnz = capacity, the count stays in row_ptr[n]): prepared and
    rebuilding calls agree, also with the call that knows the count; the gradient's tail between the end of the rows
    and nnz is zero."""
    import torch
    wl = WORKLOADS["vit_grid_b2h3"]
    g = grf.DeviceGraph.from_host(wl.graph)
    exact = grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    bound = grf.grf_sample_async(g, torch.from_numpy(wl.f).cuda(), wl.p_halt, wl.n_walks, wl.walk_seed)
    assert bound.nnz == bound.capacity > exact.nnz
    Q, K, V = (to_dev(x) for x in wl.qkv())
    prepared = grf.grf_phi_prepare(bound)
    got = grf.grf_masked_linear_attention_fused_prepared(Q, K, V, bound, prepared, return_num_den=True)
    assert all(same(a, b) for a, b in zip(got, grf.grf_masked_linear_attention_fused(Q, K, V, bound, return_num_den=True)))
    assert all(same(a, b) for a, b in zip(got, grf.grf_masked_linear_attention_fused(Q, K, V, exact, return_num_den=True)))
    out, _, den = got
    d_out = torch.randn(out.shape, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(2))
    grads = grf.grf_masked_linear_attention_backward_prepared(Q, K, V, bound, prepared, out, den, d_out)
    grads_exact = grf.grf_masked_linear_attention_backward(Q, K, V, exact, out, den, d_out)
    for a, b in zip(grads[:3], grads_exact[:3]):
        assert same(a, b)
    assert same(grads[3][:, : exact.nnz], grads_exact[3][:, : exact.nnz])
    assert torch.all(grads[3][:, exact.nnz:] == 0)      # also with the asymmetric estimator's backward
    agrads = grf.grf_asymmetric_masked_attention_backward(Q, K, V, bound, out, den, d_out)
    assert torch.all(agrads[3][:, exact.nnz:] == 0)


def test_prepared_buffer_too_small_is_refused(grf):
    import torch
    wl = WORKLOADS["tiny_grid_d32"]
    g = grf.DeviceGraph.from_host(wl.graph)
    phi = grf.grf_sample(g, wl.f, wl.p_halt, wl.n_walks, wl.walk_seed)
    Q, K, V = (to_dev(x) for x in wl.qkv())
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(grf.GrfError) as e:
        grf.grf_phi_prepare(phi, out=small)
    assert e.value.status == grf.GRF_EWORKSPACE
    with pytest.raises(grf.GrfError) as e:
        grf.grf_masked_linear_attention_fused_prepared(Q, K, V, phi, small)
    assert e.value.status == grf.GRF_EWORKSPACE


def test_training_step_over_frozen_walks_replays_from_a_hip_graph(grf):
    """The use the prepared lists are for (Sec. 4: walks frozen, f learnable): per step the values of Phi_hat follow f
    (grf_sample_async over the same walks), the prepared buffer takes them over (grf_phi_prepare_values), then the
    fused forward, the backward and the sampler's backward run over the prepared lists.  Captured once into a HIP graph
    (nothing in it touches the host) and replayed with other f: the bits of the eager, rebuilding calls every time."""
    import torch
    rng = np.random.default_rng(33)
    g_host = synth.grid_graph(24, 24, 8)
    n, n_walks, f_len, p_halt, seed = g_host.n, 8, 10, 0.5, 5
    g = grf.DeviceGraph.from_host(g_host)
    f_h = [np.abs(synth.modulation(f_len, rng, n_f=2)) + 0.01 for _ in range(3)]      # positive: no vanishing denominators
    f = torch.from_numpy(f_h[0]).cuda()
    Q, K, V = (to_dev(x) for x in synth.qkv(2, 2, n, 64, rng))
    d_out = torch.randn(Q.shape, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(3))
    phi = grf.grf_sample_async(g, f, p_halt, n_walks, seed)
    sws = torch.empty(4096, dtype=torch.uint8, device="cuda:0")
    prepared = grf.grf_phi_prepare(phi)
    prep_bytes = grf.grf_phi_prepare_bytes(n, phi.nnz, phi.n_f)
    fws = torch.empty(grf.grf_fused_attention_workspace_bytes(2, 2, n, 64, phi.nnz, 2) - prep_bytes, dtype=torch.uint8, device="cuda:0")
    bws = torch.empty(grf.grf_attention_backward_workspace_bytes(2, 2, n, 64, phi.nnz, 2) - prep_bytes, dtype=torch.uint8, device="cuda:0")
    results = {}

    def step():
        grf.grf_sample_async(g, f, p_halt, n_walks, seed, out=phi, workspace=sws)
        grf.grf_phi_prepare_values(phi, prepared)
        out, _, den = grf.grf_masked_linear_attention_fused(Q, K, V, phi, "elu1", workspace=fws, prepared=prepared, return_num_den=True)
        dQ, dK, dV, dphi = grf.grf_masked_linear_attention_backward(Q, K, V, phi, out, den, d_out, "elu1", workspace=bws, prepared=prepared)
        df = grf.grf_sample_backward(g, f_len, p_halt, n_walks, seed, phi, dphi)
        results["got"] = (out, dQ, dK, dV, df)

    def reference(ff):
        ph = grf.grf_sample(g, ff, p_halt, n_walks, seed)
        out, _, den = grf.grf_masked_linear_attention_fused(Q, K, V, ph, "elu1", return_num_den=True)
        dQ, dK, dV, dphi = grf.grf_masked_linear_attention_backward(Q, K, V, ph, out, den, d_out, "elu1")
        return out, dQ, dK, dV, grf.grf_sample_backward(g, f_len, p_halt, n_walks, seed, ph, dphi)

    step()
    torch.cuda.synchronize()
    for a, b in zip(results["got"], reference(f_h[0])):
        assert same(a, b)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    captured = results["got"]
    for trial in (1, 2, 0, 1):
        f.copy_(torch.from_numpy(f_h[trial]).cuda())
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in captured]
        for a, b in zip(got, reference(f_h[trial])):
            assert same(a, b), trial
