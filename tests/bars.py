"""The two bars of the GPU parity tests.

Normwise: max|x - ref| / max|ref| per tensor (1e-5 in fp32, 2e-2 with bf16 inputs).
Element-wise: |x - ref| <= tol |ref| + floor * mag, where mag is the same sum with every term replaced by its magnitude
(computed by the checker on |inputs|): relative to the element itself, plus a few units of rounding of what was actually
summed.  A purely relative element-wise bar is meaningless on sums that cancel; the normwise bar alone lets a small
row or bucket be wrong by its whole size.
"""
import numpy as np

FLOOR_F32 = 2.0 ** -20      # 16 units in the last place of the terms' absolute sum
FLOOR_BF16 = 2.0 ** -13     # bf16 inputs: fp32 operands of the matrix instructions enter as two bf16 pieces (2^-16 each)


def relerr(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max() if ref.size else 0.0
    return float(np.abs(x - ref).max() / scale) if scale > 0 else float(np.abs(x).max() if x.size else 0.0)


def elementwise_excess(x, ref, mag, tol, floor):
    """Largest ratio error / allowance over the elements (<= 1 passes)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    allow = tol * np.abs(ref) + floor * np.abs(np.asarray(mag, dtype=np.float64))
    err = np.abs(x - ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(err > 0, err / allow, 0.0)
    return float(ratio.max()) if ratio.size else 0.0


def magnitude_inputs(Q, K, V, val, feature_map_name):
    """Inputs whose checker result is the sum of the magnitudes of the terms of the attention sums: |V| and |Phi_hat|,
    and |Q|, |K| under the identity map (ReLU and elu + 1 are non-negative already)."""
    if feature_map_name == "identity":
        return np.abs(Q), np.abs(K), np.abs(V), np.abs(val)
    return Q, K, np.abs(V), np.abs(val)
