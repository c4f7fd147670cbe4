"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, sizes its workspaces sensibly and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "grf.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2410_03462_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2410_03462_amd import build
        build.build(verbose=False)
    b.lib()
    return b


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(grf_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_functions_are_exported(binding):
    names = declared_functions()
    assert {"grf_sample", "grf_sample_walks", "grf_masked_linear_attention", "grf_form_buckets",
            "grf_last_error"} <= set(names)
    L = binding.lib()
    for name in names:
        assert hasattr(L, name), f"{name} declared in grf.h but not exported"


def test_binding_exposes_the_same_names(binding):
    for name in declared_functions():
        if name in ("grf_last_error", "grf_sample_workspace_bytes", "grf_sample_backward_workspace_bytes"):
            continue      # used inside the binding; not user-facing
        assert hasattr(binding, name), name


def test_size_queries(binding):
    L = binding.lib()
    assert L.grf_sample_nnz_bound(256, 4, 8) == 256 * (1 + 4 * 7)
    assert L.grf_sample_nnz_bound(-1, 4, 8) == -1
    assert L.grf_sample_nnz_bound(10, 0, 8) == -1
    assert L.grf_bucket_record_floats(64) == 64 * 65
    assert L.grf_bucket_record_floats(32) == 32 * 33
    assert L.grf_bucket_record_floats(48) == -1
    ws = L.grf_sample_workspace_bytes(1000, 8, 10, 2)
    assert ws >= 2 * 10 * 4 + 8 and ws % 256 == 0
    assert L.grf_sample_workspace_bytes(1000, 0, 10, 2) == 0
    n, nnz, d = 32768, 2_440_000, 64
    all_heads = L.grf_attention_workspace_bytes(1, 8, n, d, nnz, 1, 0)
    one_head = L.grf_attention_workspace_bytes(1, 8, n, d, nnz, 1, 1)
    per_head = n * (d * d + d) * 4
    assert all_heads % 256 == 0 and one_head % 256 == 0
    assert all_heads - one_head == 7 * per_head
    assert one_head - per_head == L.grf_buckets_workspace_bytes(n, nnz, 1)
    assert one_head - per_head >= (n + 6 * nnz) * 4
    assert L.grf_buckets_workspace_bytes(n, nnz, 8) - L.grf_buckets_workspace_bytes(n, nnz, 1) >= 7 * nnz * 4
    assert L.grf_attention_workspace_bytes(1, 8, n, 48, nnz, 1, 0) == 0


def test_argument_validation_precedes_device_work(binding):
    """These calls must fail on the host, before any HIP call (there is no GPU here)."""
    L = binding.lib()
    nnz = ctypes.c_int64(0)
    st = L.grf_sample(None, None, 8, 1, 0.5, 4, 0, None, 0, None, None, ctypes.byref(nnz))
    assert st == binding.GRF_EINVAL
    assert b"graph" in L.grf_last_error()
    g = binding._Graph(10, 0, None, None, None)
    st = L.grf_sample_walks(ctypes.byref(g), 0.5, 4, 8, 0, None, None)
    assert st == binding.GRF_EINVAL          # row_ptr NULL
    phi = binding._Phi(10, 0, None, None, None)
    st = L.grf_masked_linear_attention(None, None, None, 0, 1, 1, 10, 48, ctypes.byref(phi), 0, 1, 0, 0,
                                       None, 0, None, None, None, None)
    assert st == binding.GRF_EUNSUPPORTED
    assert b"d=48" in L.grf_last_error()
    st = L.grf_masked_linear_attention(None, None, None, 7, 1, 1, 10, 64, ctypes.byref(phi), 0, 1, 0, 0,
                                       None, 0, None, None, None, None)
    assert st == binding.GRF_EINVAL
    # B*H*n beyond what one launch (and the device) covers, including products that overflow 64 bits
    for B, H in ((1 << 20, 1 << 20), (1 << 40, 1 << 40), (1 << 16, 1 << 12)):
        st = L.grf_masked_linear_attention_fused(None, None, None, 0, B, H, 10, 64, ctypes.byref(phi), 0, 1, 0, 0,
                                                 None, 0, None, None, None, None)
        assert st == binding.GRF_EUNSUPPORTED, (B, H)
        assert b"2^31" in L.grf_last_error()


def test_product_path_has_no_cpu_fallback(binding):
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_2410_03462_amd import synth
    with pytest.raises(RuntimeError):
        binding.DeviceGraph.from_host(synth.ring_graph(8))
