// Masked linear attention with asymmetric graph random features (App. D, Alg. 2).
//
// The keys take the one-hot graph feature (f^(2) = delta_0, Phi^(2) = I), so the mask estimate is
// the sampled matrix itself, M_hat = Phi_hat (sampled with f = alpha), and
//     num_i = sum_j Phi_hat[i,j] (phi(q_i) . phi(k_j)) v_j,   den_i = sum_j Phi_hat[i,j] (phi(q_i) . phi(k_j)),
// a sampled dense-dense product followed by a sparse-dense product over the CSR rows.  There are
// no buckets and no workspace.  The appendix loops over walks; summing a row's deposits per end
// node first (which is what Phi_hat holds) gives the same sums.
//
// One wavefront per (slice, row i).  d/4 lanes share one entry: each holds four features of phi(q_i),
// loads the matching 16 bytes of k_j and of v_j, the dot product is reduced over the d/4 lanes, and
// 256/d entries are in flight per step.
#include "attention_common.hpp"

namespace grf {

template <typename T>
__device__ __forceinline__ float4 load4(const T* __restrict__ p)
{
    if constexpr (sizeof(T) == 4) {
        return *reinterpret_cast<const float4*>(p);
    } else {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                           __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
    }
}

template <int D, typename T>
__global__ __launch_bounds__(256) void asymmetric_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                         long long n, int H, int n_f, long long val_stride,
                                                         const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                         const float* __restrict__ phi_val, int fmap, long long n_waves, int32_t nnz,
                                                         float* __restrict__ out, float* __restrict__ num_opt, float* __restrict__ den_opt)
{
    constexpr int LPE = D / 4;            // lanes per entry
    constexpr int EPS = kWave / LPE;      // entries per step
    constexpr int UNROLL = 4;
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long bh = wave / n;
    const long long i = wave - bh * n;
    const long long plane = n_f > 1 ? (bh % H) : 0;
    const float* vals = phi_val + plane * val_stride;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;

    const int lane = lane_id();
    const int sub = lane / LPE;
    const int cg = lane % LPE;

    float4 q4 = load4(Q + (bh * n + i) * D + 4 * cg);
    q4.x = feature(q4.x, fmap); q4.y = feature(q4.y, fmap); q4.z = feature(q4.z, fmap); q4.w = feature(q4.w, fmap);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float dacc = 0.0f;
    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        int32_t c_reg = 0;
        float w_reg = 0.0f;
        if (e < end) {
            const int32_t c = col[e];
            if (static_cast<uint32_t>(c) < static_cast<uint32_t>(n)) { c_reg = c; w_reg = vals[e]; }
        }
        const int cnt = min(kWave, end - chunk);
        // lanes past the end of the row carry column 0 with weight 0; the shuffles run in every lane
        for (int t0 = 0; t0 < cnt; t0 += EPS * UNROLL) {
            float4 k4[UNROLL], v4[UNROLL];
            float w[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int t = (t0 + u * EPS + sub) & (kWave - 1);
                const long long j = __shfl(c_reg, t, kWave);
                const float wt = __shfl(w_reg, t, kWave);     // unconditional: a masked-off source lane reads as 0
                w[u] = t0 + u * EPS + sub < cnt ? wt : 0.0f;
                k4[u] = load4(Kb + j * D + 4 * cg);
                v4[u] = load4(Vb + j * D + 4 * cg);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float p = q4.x * feature(k4[u].x, fmap);
                p = fmaf(q4.y, feature(k4[u].y, fmap), p);
                p = fmaf(q4.z, feature(k4[u].z, fmap), p);
                p = fmaf(q4.w, feature(k4[u].w, fmap), p);
                if constexpr (LPE == 16) {
                    p = row_sum16(p);
                } else {
#pragma unroll
                    for (int off = 1; off < LPE; off <<= 1) p += __shfl_xor(p, off, kWave);
                }
                const float a = w[u] * p;
                acc.x = fmaf(a, v4[u].x, acc.x);
                acc.y = fmaf(a, v4[u].y, acc.y);
                acc.z = fmaf(a, v4[u].z, acc.z);
                acc.w = fmaf(a, v4[u].w, acc.w);
                dacc += a;
            }
        }
    }
#pragma unroll
    for (int off = LPE; off < kWave; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, kWave);
        acc.y += __shfl_xor(acc.y, off, kWave);
        acc.z += __shfl_xor(acc.z, off, kWave);
        acc.w += __shfl_xor(acc.w, off, kWave);
        dacc += __shfl_xor(dacc, off, kWave);
    }
    if (sub == 0) {
        const long long o = (bh * n + i) * D + 4 * cg;
        *reinterpret_cast<float4*>(out + o) = make_float4(acc.x / dacc, acc.y / dacc, acc.z / dacc, acc.w / dacc);
        if (num_opt != nullptr) *reinterpret_cast<float4*>(num_opt + o) = acc;
        if (cg == 0 && den_opt != nullptr) den_opt[bh * n + i] = dacc;
    }
}

// ------------------------------------------------------------------------------------ gradients
// With g_i = d_out_i / den_i, a_ij = phi(q_i) . phi(k_j) and c_ij = g_i . (v_j - out_i), the loss depends on the
// inputs through sum_(i,j) Phi_ij a_ij c_ij:
//     dPhi_ij = a_ij c_ij      dphi(q_i) = sum_j Phi_ij c_ij phi(k_j)
//     dphi(k_j) = sum_i Phi_ij c_ij phi(q_i)      dv_j = sum_i Phi_ij a_ij g_i
// The first two are sums over a row of Phi_hat (rows kernel, which also leaves Phi_ij c_ij and Phi_ij a_ij per
// entry), the last two over a column (columns kernel, over the column lists, rows ascending: fixed order).

// One wavefront per (slice, row i); lanes as in the forward kernel.
template <int D, typename T>
__global__ __launch_bounds__(256) void asymmetric_backward_rows_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                                       const float* __restrict__ G, const float* __restrict__ out,
                                                                       long long n, int H, int n_f, long long val_stride,
                                                                       const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                                       const float* __restrict__ phi_val, int fmap, long long bh_first,
                                                                       long long n_waves, int32_t nnz, float* __restrict__ dQ,
                                                                       float* __restrict__ wc_out, float* __restrict__ wa_out,
                                                                       float* __restrict__ dphi_part)
{
    constexpr int LPE = D / 4;
    constexpr int EPS = kWave / LPE;
    constexpr int UNROLL = 4;
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long i = wave - slice * n;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (bh % H) : 0;
    const float* vals = phi_val + plane * val_stride;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;
    const long long ebase = slice * static_cast<long long>(nnz);

    const int lane = lane_id();
    const int sub = lane / LPE;
    const int cg = lane % LPE;

    const float4 q4 = load4(Q + (bh * n + i) * D + 4 * cg);
    const float4 fq = make_float4(feature(q4.x, fmap), feature(q4.y, fmap), feature(q4.z, fmap), feature(q4.w, fmap));
    const float4 g4 = *reinterpret_cast<const float4*>(G + (slice * n + i) * D + 4 * cg);
    // c_ij = g_i . (v_j - out_i): the difference is taken before the product, so that a row whose output is (nearly)
    // one of its values loses nothing to cancellation between two dot products
    const float4 o4 = *reinterpret_cast<const float4*>(out + (bh * n + i) * D + 4 * cg);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        int32_t c_reg = 0;
        float w_reg = 0.0f;
        if (e < end) {
            const int32_t c = col[e];
            if (static_cast<uint32_t>(c) < static_cast<uint32_t>(n)) { c_reg = c; w_reg = vals[e]; }
        }
        const int cnt = min(kWave, end - chunk);
        for (int t0 = 0; t0 < cnt; t0 += EPS * UNROLL) {
            float4 k4[UNROLL], v4[UNROLL];
            float w[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int t = (t0 + u * EPS + sub) & (kWave - 1);
                const long long j = __shfl(c_reg, t, kWave);
                const float wt = __shfl(w_reg, t, kWave);
                w[u] = t0 + u * EPS + sub < cnt ? wt : 0.0f;
                k4[u] = load4(Kb + j * D + 4 * cg);
                v4[u] = load4(Vb + j * D + 4 * cg);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float4 fk = make_float4(feature(k4[u].x, fmap), feature(k4[u].y, fmap), feature(k4[u].z, fmap), feature(k4[u].w, fmap));
                float a = fq.x * fk.x;
                a = fmaf(fq.y, fk.y, a); a = fmaf(fq.z, fk.z, a); a = fmaf(fq.w, fk.w, a);
                float c = g4.x * (v4[u].x - o4.x);
                c = fmaf(g4.y, v4[u].y - o4.y, c); c = fmaf(g4.z, v4[u].z - o4.z, c); c = fmaf(g4.w, v4[u].w - o4.w, c);
                if constexpr (LPE == 16) {
                    a = row_sum16(a);
                    c = row_sum16(c);
                } else {
#pragma unroll
                    for (int off = 1; off < LPE; off <<= 1) {
                        a += __shfl_xor(a, off, kWave);
                        c += __shfl_xor(c, off, kWave);
                    }
                }
                const float wc = w[u] * c;
                acc.x = fmaf(wc, fk.x, acc.x);
                acc.y = fmaf(wc, fk.y, acc.y);
                acc.z = fmaf(wc, fk.z, acc.z);
                acc.w = fmaf(wc, fk.w, acc.w);
                const int t = t0 + u * EPS + sub;
                if (cg == 0 && t < cnt) {
                    dphi_part[ebase + chunk + t] = a * c;
                    wc_out[ebase + chunk + t] = wc;
                    wa_out[ebase + chunk + t] = w[u] * a;
                }
            }
        }
    }
#pragma unroll
    for (int off = LPE; off < kWave; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, kWave);
        acc.y += __shfl_xor(acc.y, off, kWave);
        acc.z += __shfl_xor(acc.z, off, kWave);
        acc.w += __shfl_xor(acc.w, off, kWave);
    }
    if (sub == 0) {
        const long long o = (bh * n + i) * D + 4 * cg;
        *reinterpret_cast<float4*>(dQ + o) = make_float4(acc.x * feature_grad(q4.x, fmap), acc.y * feature_grad(q4.y, fmap),
                                                         acc.z * feature_grad(q4.z, fmap), acc.w * feature_grad(q4.w, fmap));
    }
}

// One wavefront per (slice, column j) over the column list of j (rows ascending).
template <int D, typename T>
__global__ __launch_bounds__(256) void asymmetric_backward_columns_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                                                                          const float* __restrict__ G, long long n,
                                                                          const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row,
                                                                          const int32_t* __restrict__ csc_src,
                                                                          const float* __restrict__ wc_in, const float* __restrict__ wa_in,
                                                                          int fmap, long long bh_first, long long n_waves, int32_t nnz,
                                                                          float* __restrict__ dK, float* __restrict__ dV)
{
    constexpr int LPE = D / 4;
    constexpr int EPS = kWave / LPE;
    constexpr int UNROLL = 4;
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long j = wave - slice * n;
    const long long bh = bh_first + slice;
    const T* Qb = Q + bh * n * D;
    const float* Gb = G + slice * n * D;
    const long long ebase = slice * static_cast<long long>(nnz);

    const int lane = lane_id();
    const int sub = lane / LPE;
    const int cg = lane % LPE;

    float4 acck = make_float4(0.f, 0.f, 0.f, 0.f), accv = make_float4(0.f, 0.f, 0.f, 0.f);
    const int32_t beg = col_ptr[j];
    const int32_t end = col_ptr[j + 1];
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        int32_t i_reg = 0;
        float wc_reg = 0.0f, wa_reg = 0.0f;
        if (e < end) {
            i_reg = csc_row[e];
            const int32_t src = csc_src[e];
            wc_reg = wc_in[ebase + src];
            wa_reg = wa_in[ebase + src];
        }
        const int cnt = min(kWave, end - chunk);
        for (int t0 = 0; t0 < cnt; t0 += EPS * UNROLL) {
            float4 q4[UNROLL], g4[UNROLL];
            float wc[UNROLL], wa[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int t = (t0 + u * EPS + sub) & (kWave - 1);
                const long long i = __shfl(i_reg, t, kWave);
                const float c1 = __shfl(wc_reg, t, kWave), a1 = __shfl(wa_reg, t, kWave);
                const bool ok = t0 + u * EPS + sub < cnt;
                wc[u] = ok ? c1 : 0.0f;
                wa[u] = ok ? a1 : 0.0f;
                q4[u] = load4(Qb + i * D + 4 * cg);
                g4[u] = *reinterpret_cast<const float4*>(Gb + i * D + 4 * cg);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                acck.x = fmaf(wc[u], feature(q4[u].x, fmap), acck.x);
                acck.y = fmaf(wc[u], feature(q4[u].y, fmap), acck.y);
                acck.z = fmaf(wc[u], feature(q4[u].z, fmap), acck.z);
                acck.w = fmaf(wc[u], feature(q4[u].w, fmap), acck.w);
                accv.x = fmaf(wa[u], g4[u].x, accv.x);
                accv.y = fmaf(wa[u], g4[u].y, accv.y);
                accv.z = fmaf(wa[u], g4[u].z, accv.z);
                accv.w = fmaf(wa[u], g4[u].w, accv.w);
            }
        }
    }
#pragma unroll
    for (int off = LPE; off < kWave; off <<= 1) {
        acck.x += __shfl_xor(acck.x, off, kWave); acck.y += __shfl_xor(acck.y, off, kWave);
        acck.z += __shfl_xor(acck.z, off, kWave); acck.w += __shfl_xor(acck.w, off, kWave);
        accv.x += __shfl_xor(accv.x, off, kWave); accv.y += __shfl_xor(accv.y, off, kWave);
        accv.z += __shfl_xor(accv.z, off, kWave); accv.w += __shfl_xor(accv.w, off, kWave);
    }
    if (sub == 0) {
        const long long o = (bh * n + j) * D + 4 * cg;
        const float4 k4 = load4(K + o);
        *reinterpret_cast<float4*>(dK + o) = make_float4(acck.x * feature_grad(k4.x, fmap), acck.y * feature_grad(k4.y, fmap),
                                                         acck.z * feature_grad(k4.z, fmap), acck.w * feature_grad(k4.w, fmap));
        *reinterpret_cast<float4*>(dV + o) = accv;
    }
}

namespace {

struct AsymmetricScratch {
    float* G;        // [chunk][n][d]
    float* gd;       // [chunk][n]
    float* wc;       // [chunk][nnz]  Phi_ij c_ij, CSR order
    float* wa;       // [chunk][nnz]  Phi_ij a_ij
    float* dpart;    // [chunk][nnz]  a_ij c_ij
    size_t bytes;
};

AsymmetricScratch carve_asymmetric(unsigned char* ws, int64_t slices, int64_t n, int32_t d, int64_t nnz)
{
    AsymmetricScratch b;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = ws ? ws + off : nullptr; off += align_up(bytes); return reinterpret_cast<float*>(p); };
    const size_t entries = static_cast<size_t>(nnz > 0 ? nnz : 1), rows = static_cast<size_t>(n > 0 ? n : 1), sl = static_cast<size_t>(slices > 0 ? slices : 1);
    b.G = take(sizeof(float) * sl * rows * d);
    b.gd = take(sizeof(float) * sl * rows);
    b.wc = take(sizeof(float) * sl * entries);
    b.wa = take(sizeof(float) * sl * entries);
    b.dpart = take(sizeof(float) * sl * entries);
    b.bytes = off;
    return b;
}

template <int D, typename T>
grf_status launch_asymmetric_backward_chunk(const void* Qv, const void* Kv, const void* Vv, int64_t n, int64_t H, int32_t n_f,
                                            const grf_phi* phi, int64_t nnz, const Transposed& t, const AsymmetricScratch& b, int fmap,
                                            int64_t bh_first, int64_t n_slices, const float* out, const float* den, const float* d_out,
                                            float* dQ, float* dK, float* dV, float* dphi_val, hipStream_t stream)
{
    const T* Q = static_cast<const T*>(Qv);
    const T* K = static_cast<const T*>(Kv);
    const T* V = static_cast<const T*>(Vv);
    const long long waves = static_cast<long long>(n_slices) * n;
    if (waves == 0) return GRF_OK;
    if (grf_status st = launch_backward_seed(D, out, den, d_out, static_cast<long long>(bh_first) * n, waves, b.G, b.gd, stream)) return st;
    hipLaunchKernelGGL((asymmetric_backward_rows_kernel<D, T>), dim3(blocks_for(waves, 4)), dim3(256), 0, stream, Q, K, V,
                       static_cast<const float*>(b.G), out, static_cast<long long>(n), static_cast<int>(H),
                       static_cast<int>(n_f), static_cast<long long>(phi->capacity), static_cast<const int32_t*>(phi->row_ptr),
                       static_cast<const int32_t*>(phi->col), static_cast<const float*>(phi->val), fmap,
                       static_cast<long long>(bh_first), waves, static_cast<int32_t>(nnz), dQ, b.wc, b.wa, b.dpart);
    GRF_LAUNCH_CHECK("asymmetric_backward_rows_kernel");
    hipLaunchKernelGGL((asymmetric_backward_columns_kernel<D, T>), dim3(blocks_for(waves, 4)), dim3(256), 0, stream, Q, K,
                       static_cast<const float*>(b.G), static_cast<long long>(n), static_cast<const int32_t*>(t.col_ptr),
                       static_cast<const int32_t*>(t.s_row), static_cast<const int32_t*>(t.s_src),
                       static_cast<const float*>(b.wc), static_cast<const float*>(b.wa), fmap, static_cast<long long>(bh_first),
                       waves, static_cast<int32_t>(nnz), dK, dV);
    GRF_LAUNCH_CHECK("asymmetric_backward_columns_kernel");
    return launch_dphi_accumulate(nnz, n_f, H, bh_first, n_slices, b.dpart, nullptr, phi, dphi_val, stream);
}

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" grf_status grf_asymmetric_masked_attention(const void* Q, const void* K, const void* V, int32_t dtype,
                                                      int64_t B, int64_t H, int64_t n, int32_t d,
                                                      const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                      void* hip_stream, float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr)) return fail(GRF_EINVAL, "Q / out is NULL");
    if (B * H * n == 0) return GRF_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int fmap = feature_map;
    const long long waves = static_cast<long long>(B) * H * n;
    GRF_DISPATCH(d, dtype,
                 hipLaunchKernelGGL((asymmetric_kernel<D_, T_>), dim3(blocks_for(waves, 4)), dim3(256), 0, stream,
                                    static_cast<const T_*>(Q), static_cast<const T_*>(K), static_cast<const T_*>(V),
                                    static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f),
                                    static_cast<long long>(phi->capacity), static_cast<const int32_t*>(phi->row_ptr),
                                    static_cast<const int32_t*>(phi->col), static_cast<const float*>(phi->val), fmap, waves,
                                    static_cast<int32_t>(nnz), out, num_opt, den_opt));
    GRF_LAUNCH_CHECK("asymmetric_kernel");
    return GRF_OK;
}

extern "C" size_t grf_asymmetric_backward_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk)
{
    if (B < 0 || H < 0 || n < 0 || nnz < 0 || n_f < 1 || (d != 32 && d != 64)) return 0;
    int64_t slices = B * H;
    if (bh_chunk > 0 && bh_chunk < slices) slices = bh_chunk;
    return carve_transposed(nullptr, n, nnz, n_f).bytes + carve_asymmetric(nullptr, slices, n, d, nnz).bytes;
}

extern "C" grf_status grf_asymmetric_masked_attention_backward(const void* Q, const void* K, const void* V, int32_t dtype,
                                                               int64_t B, int64_t H, int64_t n, int32_t d,
                                                               const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                               const float* out, const float* den, const float* d_out,
                                                               int32_t bh_chunk,
                                                               void* workspace, size_t workspace_bytes, void* hip_stream,
                                                               float* dQ, float* dK, float* dV, float* dphi_val)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr || den == nullptr || d_out == nullptr))
        return fail(GRF_EINVAL, "Q / out / den / d_out is NULL");
    if (B * H * n > 0 && (dQ == nullptr || dK == nullptr || dV == nullptr)) return fail(GRF_EINVAL, "dQ / dK / dV is NULL");
    if (grf_status st = check_workspace(workspace, workspace_bytes, grf_asymmetric_backward_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B * H * n == 0) {
        if (dphi_val != nullptr && nnz > 0)
            for (int32_t h = 0; h < n_f; ++h)
                if (grf_status st = fill_i32(reinterpret_cast<int32_t*>(dphi_val + static_cast<int64_t>(h) * phi->capacity), nnz, 0, stream)) return st;
        return GRF_OK;
    }
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const Transposed t = carve_transposed(ws, n, nnz, n_f);
    const AsymmetricScratch b = carve_asymmetric(ws + t.bytes, step, n, d, nnz);
    if (grf_status st = transpose(phi, nnz, n_f, t, stream)) return st;
    for (int64_t first = 0; first < slices; first += step) {
        const int64_t count = (slices - first < step) ? (slices - first) : step;
        grf_status st = GRF_OK;
        GRF_DISPATCH(d, dtype, (st = launch_asymmetric_backward_chunk<D_, T_>(Q, K, V, n, H, n_f, phi, nnz, t, b, feature_map, first, count,
                                                                              out, den, d_out, dQ, dK, dV, dphi_val, stream)));
        if (st != GRF_OK) return st;
    }
    return GRF_OK;
}
