"""CPU checker for GRF-masked linear attention (arXiv 2410.03462) -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``grf_oracle.c`` plus the dense, quadratic definitions in
numpy that the C routines are themselves pinned against.  Nothing here is used by
the HIP library and nothing here imports it.  Only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this module.

All routines take and return numpy arrays on the host; accumulation is fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "grf_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libgrf_oracle.so")
_lib = None

RELU, IDENTITY, ELU1 = 0, 1, 2


_SAN_LIB_PATH = os.path.join(_HERE, "libgrf_oracle_san.so")


def sanitized() -> bool:
    """True when GRF_ORACLE_SANITIZE=1 selects the build with AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

    The sanitizer runtime has to be in the process before Python starts:
        GRF_ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 LD_PRELOAD=$(gcc -print-file-name=libasan.so) \
            python -m pytest tests -m "not gpu"
    Any invalid access or undefined operation inside the checker then aborts the run with a report."""
    return os.environ.get("GRF_ORACLE_SANITIZE", "") == "1"


def build(force: bool = False, sanitize: bool = None) -> str:
    """Compile grf_oracle.c with gcc (-O2, no fast-math); ``sanitize`` (default: sanitized()) adds
    -fsanitize=address,undefined and writes a library of its own."""
    sanitize = sanitized() if sanitize is None else sanitize
    path = _SAN_LIB_PATH if sanitize else _LIB_PATH
    if force or not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if sanitize else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-o", path, _SRC, "-lm"])
    return path


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.grf_ref_sample.restype = ctypes.c_int64
        _lib.grf_ref_dphi_entry_direct.restype = ctypes.c_double
        _lib.grf_ref_knn_graph.restype = ctypes.c_int64
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


# --------------------------------------------------------------------------- random stream

def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    _load().grf_ref_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


# --------------------------------------------------------------------------- walks and features

def sample_walks(g, p_halt: float, n_walks: int, max_nodes: int, seed: int, with_loads: bool = False):
    """Trajectories [n, n_walks, max_nodes] (int32, -1 padded) and optionally the fp64 loads."""
    traj = np.empty((g.n, n_walks, max_nodes), dtype=np.int32)
    loads = np.empty((g.n, n_walks, max_nodes), dtype=np.float64) if with_loads else None
    rp, col, w = _i32(g.row_ptr), _i32(g.col), _f32(g.w)
    _load().grf_ref_sample_walks(
        ctypes.c_int64(g.n), _p(rp, ctypes.c_int32), _p(col, ctypes.c_int32), _p(w, ctypes.c_float),
        ctypes.c_double(p_halt), ctypes.c_int32(n_walks), ctypes.c_int32(max_nodes), ctypes.c_uint64(seed),
        _p(traj, ctypes.c_int32), _p(loads, ctypes.c_double))
    return (traj, loads) if with_loads else traj


def sample(g, f, p_halt: float, n_walks: int, seed: int):
    """GRF matrix Phi_hat in CSR: (row_ptr int32[n+1], col int32[nnz], val float32[n_f, nnz])."""
    f = _f32(np.atleast_2d(f))
    n_f, f_len = f.shape
    rp, col, w = _i32(g.row_ptr), _i32(g.col), _f32(g.w)
    row_ptr = np.zeros(g.n + 1, dtype=np.int32)
    lib = _load()

    def call(col_out, val_out):
        return lib.grf_ref_sample(
            ctypes.c_int64(g.n), _p(rp, ctypes.c_int32), _p(col, ctypes.c_int32), _p(w, ctypes.c_float),
            _p(f, ctypes.c_float), ctypes.c_int32(f_len), ctypes.c_int32(n_f),
            ctypes.c_double(p_halt), ctypes.c_int32(n_walks), ctypes.c_uint64(seed),
            _p(row_ptr, ctypes.c_int32), _p(col_out, ctypes.c_int32), _p(val_out, ctypes.c_float))

    nnz = call(None, None)
    col_out = np.empty(nnz, dtype=np.int32)
    val_out = np.empty((n_f, nnz), dtype=np.float32)
    call(col_out, val_out)
    return row_ptr, col_out, val_out


def phi_dense(n, row_ptr, col, val) -> np.ndarray:
    """Dense fp64 copy of one value plane of Phi_hat."""
    P = np.zeros((n, n), dtype=np.float64)
    rows = np.repeat(np.arange(n), np.diff(row_ptr))
    P[rows, col] = val.astype(np.float64)
    return P


# --------------------------------------------------------------------------- exact quantities (dense, tiny graphs)

def exact_features(W: np.ndarray, f: np.ndarray) -> np.ndarray:
    """Phi_G = sum_t f_t W^t  (Remark 3.1), dense fp64."""
    n = W.shape[0]
    P = np.eye(n)
    out = np.zeros((n, n))
    for ft in np.asarray(f, dtype=np.float64):
        out += ft * P
        P = P @ W
    return out


def exact_mask(W: np.ndarray, f: np.ndarray) -> np.ndarray:
    """M_alpha = sum_k alpha_k W^k with alpha = f * f (discrete convolution; Eq. 4, Remark 3.1)."""
    f = np.asarray(f, dtype=np.float64)
    alpha = np.convolve(f, f)
    n = W.shape[0]
    P = np.eye(n)
    out = np.zeros((n, n))
    for a in alpha:
        out += a * P
        P = P @ W
    return out


# --------------------------------------------------------------------------- attention

def _feature(x: np.ndarray, feature_map: int) -> np.ndarray:
    x = x.astype(np.float64)
    if feature_map == RELU:
        return np.maximum(x, 0.0)
    if feature_map == ELU1:          # elu(x) + 1
        return np.where(x > 0.0, x + 1.0, np.exp(np.minimum(x, 0.0)))
    return x


def attention_bruteforce(Q, K, V, M, feature_map: int = RELU):
    """Eq. (1)-(2): A_M = M .* (phi(Q) phi(K)^T); returns (num, den, out) in fp64.  One (b,h) slice."""
    A = _feature(Q, feature_map) @ _feature(K, feature_map).T
    AM = M * A
    num = AM @ V.astype(np.float64)
    den = AM.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        out = num / den[:, None]
    return num, den, out


def buckets(K, V, row_ptr, col, val, feature_map: int = RELU):
    """S [n,d,d], z [n,d] in fp64 for one (b,h) slice (Alg. 1 step 5, the Phi_K^T products)."""
    K, V = _f32(K), _f32(V)
    n, d = K.shape
    S = np.empty((n, d, d), dtype=np.float64)
    z = np.empty((n, d), dtype=np.float64)
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    _load().grf_ref_buckets(
        ctypes.c_int64(n), ctypes.c_int32(d), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(S, ctypes.c_double), _p(z, ctypes.c_double))
    return S, z


def gather(Q, row_ptr, col, val, S, z, feature_map: int = RELU):
    """num [n,d], den [n] in fp64 for one (b,h) slice (Alg. 1 step 5, the Phi_Q products)."""
    Q = _f32(Q)
    n, d = Q.shape
    num = np.empty((n, d), dtype=np.float64)
    den = np.empty(n, dtype=np.float64)
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    S = np.ascontiguousarray(S, dtype=np.float64)
    z = np.ascontiguousarray(z, dtype=np.float64)
    _load().grf_ref_gather(
        ctypes.c_int64(n), ctypes.c_int32(d), _p(Q, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(S, ctypes.c_double), _p(z, ctypes.c_double), _p(num, ctypes.c_double), _p(den, ctypes.c_double))
    return num, den


def masked_linear_attention(Q, K, V, row_ptr, col, val, feature_map: int = RELU, return_buckets: bool = False):
    """Alg. 1 steps 3-5 for Q,K,V of shape [B,H,n,d].

    ``val`` is [n_f, nnz] with n_f == 1 (shared by all heads) or n_f == H (one plane per head).
    Returns dict with fp64 ``num`` [B,H,n,d], ``den`` [B,H,n], ``out`` = num/den, and optionally
    ``S`` [B,H,n,d,d], ``z`` [B,H,n,d].
    """
    Q, K, V = (np.asarray(x, dtype=np.float32) for x in (Q, K, V))
    B, H, n, d = Q.shape
    val = np.atleast_2d(val)
    assert val.shape[0] in (1, H)
    num = np.empty((B, H, n, d), dtype=np.float64)
    den = np.empty((B, H, n), dtype=np.float64)
    Ss = np.empty((B, H, n, d, d), dtype=np.float64) if return_buckets else None
    zs = np.empty((B, H, n, d), dtype=np.float64) if return_buckets else None
    for b in range(B):
        for h in range(H):
            v = val[h if val.shape[0] > 1 else 0]
            S, z = buckets(K[b, h], V[b, h], row_ptr, col, v, feature_map)
            num[b, h], den[b, h] = gather(Q[b, h], row_ptr, col, v, S, z, feature_map)
            if return_buckets:
                Ss[b, h], zs[b, h] = S, z
    with np.errstate(divide="ignore", invalid="ignore"):
        out = num / den[..., None]
    res = {"num": num, "den": den, "out": out}
    if return_buckets:
        res["S"], res["z"] = Ss, zs
    return res


def asymmetric_attention_walks(g, f, p_halt: float, n_walks: int, seed: int, Q, K, V, feature_map: int = RELU):
    """App. D, Alg. 2 walk by walk, for Q,K,V of shape [B,H,n,d] and one modulation vector f (= alpha).

    Returns dict with fp64 ``num`` [B,H,n,d], ``den`` [B,H,n] and ``out`` = num/den.
    """
    Q, K, V = (np.ascontiguousarray(x, dtype=np.float32) for x in (Q, K, V))
    B, H, n, d = Q.shape
    f = _f32(np.asarray(f).reshape(-1))
    rp, col, w = _i32(g.row_ptr), _i32(g.col), _f32(g.w)
    num = np.empty((B, H, n, d), dtype=np.float64)
    den = np.empty((B, H, n), dtype=np.float64)
    lib = _load()
    for b in range(B):
        for h in range(H):
            nb = np.empty((n, d), dtype=np.float64)
            db = np.empty(n, dtype=np.float64)
            lib.grf_ref_asymmetric_walks(
                ctypes.c_int64(n), _p(rp, ctypes.c_int32), _p(col, ctypes.c_int32), _p(w, ctypes.c_float),
                _p(f, ctypes.c_float), ctypes.c_int32(f.shape[0]), ctypes.c_double(p_halt), ctypes.c_int32(n_walks),
                ctypes.c_uint64(seed), ctypes.c_int32(d),
                _p(Q[b, h], ctypes.c_float), _p(K[b, h], ctypes.c_float), _p(V[b, h], ctypes.c_float),
                ctypes.c_int32(feature_map), _p(nb, ctypes.c_double), _p(db, ctypes.c_double))
            num[b, h], den[b, h] = nb, db
    with np.errstate(divide="ignore", invalid="ignore"):
        out = num / den[..., None]
    return {"num": num, "den": den, "out": out}


def row_direct(i: int, Q, K, V, row_ptr, col, val, feature_map: int = RELU):
    """(num_i [d], den_i, mask_row [n]) for one query row of one (b,h) slice, from Eq. (2) directly."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    n, d = Q.shape
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    mask_row = np.empty(n, dtype=np.float64)
    num = np.empty(d, dtype=np.float64)
    den = ctypes.c_double(0.0)
    _load().grf_ref_row_direct(
        ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int64(i),
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(mask_row, ctypes.c_double), _p(num, ctypes.c_double), ctypes.byref(den))
    return num, den.value, mask_row


def conditioning_floor(Q, row_ptr, col, val, z, feature_map: int = RELU) -> np.ndarray:
    """sum_l |phi_hat_il| * |phi(q_i) . z_l| per row: the scale against which den_i is judged.

    f may be signed, so den_i can cancel to ~0 (Eq. 12 has no epsilon).  Rows with
    |den_i| below a small fraction of this scale are ill-conditioned for num/den.
    """
    n, d = Q.shape
    fq = _feature(np.asarray(Q), feature_map)
    rows = np.repeat(np.arange(n), np.diff(row_ptr))
    dots = np.abs(np.einsum("ea,ea->e", fq[rows], z[col]))
    return np.bincount(rows, weights=np.abs(val.astype(np.float64)) * dots, minlength=n)


# --------------------------------------------------------------------------- gradients (training with learnable f)

def backward_seed(out, den, dout) -> np.ndarray:
    """g' = dL/d[num, den] per row, [n, d+1] fp64, from the saved forward results of one slice:
    g'_i = [dout_i / den_i, -(dout_i . out_i) / den_i]  (chain rule through out = num / den)."""
    out = np.asarray(out, dtype=np.float64)
    den = np.asarray(den, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    return np.concatenate([dout / den[:, None], -(dout * out).sum(axis=1, keepdims=True) / den[:, None]], axis=1)


def attention_backward(Q, K, V, row_ptr, col, val, out, den, dout, feature_map: int = RELU):
    """Gradients of L = sum(dout * out) for one (b,h) slice: (dQ [n,d], dK, dV, dphi [nnz]) in fp64.

    ``out`` [n,d] and ``den`` [n] are the saved forward results (any float dtype; used in fp64)."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    n, d = Q.shape
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    out = np.ascontiguousarray(out, dtype=np.float64)
    den = np.ascontiguousarray(den, dtype=np.float64)
    dout = np.ascontiguousarray(dout, dtype=np.float64)
    dQ = np.empty((n, d), dtype=np.float64)
    dK = np.empty((n, d), dtype=np.float64)
    dV = np.empty((n, d), dtype=np.float64)
    dphi = np.empty(c.shape[0], dtype=np.float64)
    _load().grf_ref_attention_backward(
        ctypes.c_int64(n), ctypes.c_int32(d), _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(out, ctypes.c_double), _p(den, ctypes.c_double), _p(dout, ctypes.c_double),
        _p(dQ, ctypes.c_double), _p(dK, ctypes.c_double), _p(dV, ctypes.c_double), _p(dphi, ctypes.c_double))
    return dQ, dK, dV, dphi


def masked_linear_attention_backward(Q, K, V, row_ptr, col, val, out, den, dout, feature_map: int = RELU):
    """All slices of [B,H,n,d] tensors.  Returns dQ, dK, dV [B,H,n,d] and dphi [n_f, nnz]
    (summed over the slices that share a value plane), fp64."""
    Q, K, V = (np.asarray(x, dtype=np.float32) for x in (Q, K, V))
    B, H, n, d = Q.shape
    val = np.atleast_2d(val)
    n_f = val.shape[0]
    assert n_f in (1, H)
    dQ, dK, dV = (np.empty((B, H, n, d), dtype=np.float64) for _ in range(3))
    dphi = np.zeros((n_f, val.shape[1]), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            p = h if n_f > 1 else 0
            dQ[b, h], dK[b, h], dV[b, h], de = attention_backward(
                Q[b, h], K[b, h], V[b, h], row_ptr, col, val[p], out[b, h], den[b, h], dout[b, h], feature_map)
            dphi[p] += de
    return dQ, dK, dV, dphi


def sample_backward(g, f_len: int, p_halt: float, n_walks: int, seed: int, row_ptr, col, dphi) -> np.ndarray:
    """df [n_f, f_len] fp64 from dphi [n_f, nnz] (CSR order of the pattern sampled with the same arguments)."""
    dphi = np.ascontiguousarray(np.atleast_2d(dphi), dtype=np.float64)
    n_f, nnz = dphi.shape
    rp, c, w = _i32(g.row_ptr), _i32(g.col), _f32(g.w)
    prp, pc = _i32(row_ptr), _i32(col)
    df = np.empty((n_f, f_len), dtype=np.float64)
    _load().grf_ref_sample_backward(
        ctypes.c_int64(g.n), _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(w, ctypes.c_float),
        ctypes.c_int32(f_len), ctypes.c_int32(n_f), ctypes.c_double(p_halt), ctypes.c_int32(n_walks), ctypes.c_uint64(seed),
        _p(prp, ctypes.c_int32), _p(pc, ctypes.c_int32), ctypes.c_int64(nnz), _p(dphi, ctypes.c_double), _p(df, ctypes.c_double))
    return df


def row_direct_backward(i: int, Q, K, V, row_ptr, col, val, gp, feature_map: int = RELU):
    """(dq_i, dk_i, dv_i) [d] each for one node of one slice, from Eq. (2) directly; gp = backward_seed(...)."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    n, d = Q.shape
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    gp = np.ascontiguousarray(gp, dtype=np.float64)
    res = [np.empty(d, dtype=np.float64) for _ in range(3)]
    _load().grf_ref_row_direct_backward(
        ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int64(i),
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(gp, ctypes.c_double), *[_p(r, ctypes.c_double) for r in res])
    return tuple(res)


def dphi_entry_direct(i: int, l: int, Q, K, V, row_ptr, col, val, gp, feature_map: int = RELU) -> float:
    """dL/dPhi_hat[i, l] for one stored entry of one slice, its two buckets formed by a scan of column l."""
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    n, d = Q.shape
    rp, c, v = _i32(row_ptr), _i32(col), _f32(val)
    gp = np.ascontiguousarray(gp, dtype=np.float64)
    return float(_load().grf_ref_dphi_entry_direct(
        ctypes.c_int64(n), ctypes.c_int32(d), ctypes.c_int64(i), ctypes.c_int64(l),
        _p(Q, ctypes.c_float), _p(K, ctypes.c_float), _p(V, ctypes.c_float),
        _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(v, ctypes.c_float), ctypes.c_int32(feature_map),
        _p(gp, ctypes.c_double)))


def asymmetric_attention_backward(Q, K, V, row_ptr, col, val, out, den, dout, feature_map: int = RELU):
    """Gradients of asymmetric-GRF attention (App. D) for [B,H,n,d] tensors: dQ, dK, dV [B,H,n,d] and
    dphi [n_f, nnz] (summed over the slices that share a plane), fp64."""
    Q, K, V = (np.ascontiguousarray(x, dtype=np.float32) for x in (Q, K, V))
    B, H, n, d = Q.shape
    val = np.ascontiguousarray(np.atleast_2d(val), dtype=np.float32)
    n_f = val.shape[0]
    assert n_f in (1, H)
    rp, c = _i32(row_ptr), _i32(col)
    out = np.ascontiguousarray(out, dtype=np.float64)
    den = np.ascontiguousarray(den, dtype=np.float64)
    dout = np.ascontiguousarray(dout, dtype=np.float64)
    dQ, dK, dV = (np.empty((B, H, n, d), dtype=np.float64) for _ in range(3))
    dphi = np.zeros((n_f, val.shape[1]), dtype=np.float64)
    lib = _load()
    for b in range(B):
        for h in range(H):
            p = h if n_f > 1 else 0
            de = np.empty(val.shape[1], dtype=np.float64)
            lib.grf_ref_asymmetric_backward(
                ctypes.c_int64(n), ctypes.c_int32(d), _p(Q[b, h], ctypes.c_float), _p(K[b, h], ctypes.c_float),
                _p(V[b, h], ctypes.c_float), _p(rp, ctypes.c_int32), _p(c, ctypes.c_int32), _p(val[p], ctypes.c_float),
                ctypes.c_int32(feature_map), _p(out[b, h], ctypes.c_double), _p(den[b, h], ctypes.c_double),
                _p(dout[b, h], ctypes.c_double), _p(dQ[b, h], ctypes.c_double), _p(dK[b, h], ctypes.c_double),
                _p(dV[b, h], ctypes.c_double), _p(de, ctypes.c_double))
            dphi[p] += de
    return dQ, dK, dV, dphi


# --------------------------------------------------------------------------- graph construction for point clouds

WEIGHT_INV_DEGREE, WEIGHT_EXP, WEIGHT_GAUSS = 0, 1, 2


def knn_lists(points, k: int):
    """Brute-force k nearest neighbours of fp32 points [n,3]: (idx int32 [n,k], squared distances fp32 [n,k]),
    ordered by (fp32 squared distance, index); -1 / inf where fewer than k other points exist."""
    pts = _f32(points)
    n = pts.shape[0]
    idx = np.empty((n, k), dtype=np.int32)
    d2 = np.empty((n, k), dtype=np.float32)
    _load().grf_ref_knn_lists(ctypes.c_int64(n), _p(pts, ctypes.c_float), ctypes.c_int32(k), _p(idx, ctypes.c_int32), _p(d2, ctypes.c_float))
    return idx, d2


def knn_lists_rows(points, k: int, rows):
    """knn_lists for the query points ``rows`` only (brute force over all points for each)."""
    pts = _f32(points)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    idx = np.empty((len(rows), k), dtype=np.int32)
    d2 = np.empty((len(rows), k), dtype=np.float32)
    _load().grf_ref_knn_lists_rows(ctypes.c_int64(pts.shape[0]), _p(pts, ctypes.c_float), ctypes.c_int32(k), ctypes.c_int64(len(rows)),
                                   _p(rows, ctypes.c_int64), _p(idx, ctypes.c_int32), _p(d2, ctypes.c_float))
    return idx, d2


def knn_graph(points, k: int, symmetrise: bool = True, weight_kind: int = WEIGHT_GAUSS, sigma: float = 1.0):
    """(row_ptr int32 [n+1], col int32 [nnz], w float64 [nnz]) of the (symmetrised) k-nearest-neighbour graph."""
    idx, d2 = knn_lists(points, k)
    n = idx.shape[0]
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    lib = _load()

    def call(col, w):
        return lib.grf_ref_knn_graph(ctypes.c_int64(n), ctypes.c_int32(k), _p(idx, ctypes.c_int32), _p(d2, ctypes.c_float),
                                     ctypes.c_int32(1 if symmetrise else 0), ctypes.c_int32(weight_kind), ctypes.c_double(sigma),
                                     _p(row_ptr, ctypes.c_int32), _p(col, ctypes.c_int32), _p(w, ctypes.c_double))

    nnz = call(None, None)
    col = np.empty(nnz, dtype=np.int32)
    w = np.empty(nnz, dtype=np.float64)
    call(col, w)
    return row_ptr, col, w
