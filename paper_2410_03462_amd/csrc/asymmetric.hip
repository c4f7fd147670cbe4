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
#pragma unroll
                for (int off = 1; off < LPE; off <<= 1) p += __shfl_xor(p, off, kWave);
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
