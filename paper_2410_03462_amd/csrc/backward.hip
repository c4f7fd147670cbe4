// Gradients of GRF-masked linear attention (Eq. 7; Alg. 1 with learnable f) on gfx950.
//
// With v'_j = [v_j, 1], g'_i = [d_out_i / den_i, -(d_out_i . out_i) / den_i] and, per bucket l with
// contributor list C_l and weights w_i = Phi_hat[i, l],
//     S'_l = sum_j w_j phi(k_j) v'_j^T        T'_l = sum_i w_i phi(q_i) g'_i^T
// the gradients are
//     dphi(q_i) += w_i S'_l g'_i      dphi(k_i) += w_i T'_l v'_i      dv_i += w_i T_l^T phi(k_i)
//     dPhi[i,l]  = phi(q_i) . (S'_l g'_i) + phi(k_i) . (T'_l v'_i)
// for every i in C_l: as in the fused forward pass, the rows that consume a bucket are its contributors.
//
// Three passes, each one wavefront per (slice, bucket) running two MFMA contractions
// (v_mfma_f32_32x32x2_f32) like the forward kernel; a pass differs in which rows feed which operand:
//
//   pass           first contraction ACC = A^T B            second contraction, per consumer i     streams out
//   kQuerySide     A = V,        B = w phi(K), +sum B (z)    U_i = g_i ACC + gd_i z                 U_i
//   kKeySide       A = G,        B = w phi(Q), +sum gd B (y) R_i = v_i ACC + y                      R_i
//   kValueSide     A = w phi(Q), B = G                       X_i = phi(k_i) ACC                     X_i
//
// (ACC is S^T, T^T and T respectively: the second contraction always runs over the row index of ACC,
// which is the index the accumulator registers of a lane enumerate.)  A second kernel, one wavefront per
// output row, reads the row's streamed vectors in ascending-l order: it forms dphi(q_i) = sum_l w_il U_il
// (likewise k and v), and on the way the per-entry terms phi(q_i).U_il and phi(k_i).R_il of dPhi.  Sums have a fixed order: results are bitwise reproducible and no float atomics are used.
#include <type_traits>

#include "attention_common.hpp"
#include "backward_split.hpp"
#include "gram_split.hpp"

namespace grf {

// g' per row of a chunk of slices: G[s][i][:] = d_out / den, gd[s][i] = -(d_out . out) / den.
template <int D>
__global__ __launch_bounds__(256) void backward_seed_kernel(const float* __restrict__ out, const float* __restrict__ den,
                                                            const float* __restrict__ d_out, long long first_row, long long n_rows,
                                                            float* __restrict__ G, float* __restrict__ gd)
{
    constexpr int RPW = kWave / D;        // rows per wavefront
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int lane = lane_id();
    const long long r = wave * RPW + lane / D;      // row inside the chunk
    const int c = lane % D;
    const bool ok = r < n_rows;
    const long long src = (first_row + (ok ? r : 0)) * D + c;
    const float dn = den[first_row + (ok ? r : 0)];
    const float go = d_out[src];
    float dot = go * out[src];
#pragma unroll
    for (int off = 1; off < D; off <<= 1) dot += __shfl_xor(dot, off, kWave);
    if (ok) {
        G[r * D + c] = go / dn;
        if (c == 0) gd[r] = -dot / dn;
    }
}

// One wavefront per (slice, bucket l), one wavefront per workgroup.  Every global load is
// unconditional (lanes past the end of the column list re-read its last entry with weight 0).
template <int D, typename T, int MODE, bool WIDE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void backward_bucket_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                              const float* __restrict__ G, const float* __restrict__ gd,
                                                              long long n, int H, int n_f,
                                                              const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row,
                                                              const float* __restrict__ csc_val,
                                                              int fmap, long long bh_first, long long n_waves, int32_t nnz,
                                                              int spread_xcds, float* __restrict__ partial)
{
    constexpr int T2 = D / 32;
    constexpr int QN = 4 * T2;     // operand elements a lane holds per group of four accumulator registers
    if (blockIdx.x >= n_waves) return;
    const BucketId bucket = bucket_of_workgroup(n, spread_xcds);
    const uint32_t l32 = bucket.l;
    const long long slice = bucket.slice;
    const long long l = l32;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (static_cast<uint32_t>(bh) % static_cast<uint32_t>(H)) : 0u;
    const T* Qb = Q + bh * n * D;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;
    const float* Gb = G + slice * n * D;
    const float* gdb = gd + slice * n;
    const float* vals = csc_val + plane * nnz;

    const int lane = lane_id();
    const int half = lane >> 5;
    const int li = lane & 31;

    const int32_t beg = __builtin_amdgcn_readfirstlane(col_ptr[l]);
    const int32_t end = __builtin_amdgcn_readfirstlane(col_ptr[l + 1]);
    if (beg >= end) return;

    // consumers of tile `tile`: row index of entry tile + li (clamped to the last entry)
    auto fetch_index = [&](int32_t tile, int32_t& row) { row = csc_row[min(tile + li, end - 1)]; };
    // consumer li's operand elements for the accumulator rows this lane pairs with, and its coefficient of the extra row
    auto fetch_operand = [&](int32_t row, float (&cc)[4][QN], float& cf) {
        const uint32_t r = static_cast<uint32_t>(row);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int elem = T2 * (8 * b + 4 * half);
            if constexpr (MODE == kQuerySide) load_run<float, QN>(row_elem_ptr<D, float, WIDE>(Gb, r, elem), cc[b]);
            if constexpr (MODE == kKeySide) load_run<T, QN>(row_elem_ptr<D, T, WIDE>(Vb, r, elem), cc[b]);
            if constexpr (MODE == kValueSide) load_run<T, QN>(row_elem_ptr<D, T, WIDE>(Kb, r, elem), cc[b]);
        }
        if constexpr (MODE == kQuerySide) cf = gdb[row];
    };

    // the first two consumer tiles' indices and the first tile's operand rows go out before the first
    // contraction starts, so that they have arrived when it ends
    int32_t row_cur, row_next;
    fetch_index(beg, row_cur);
    fetch_index(beg + 32, row_next);
    float cn[4][QN];
    float cfn = 1.0f;
    fetch_operand(row_cur, cn, cfn);

    // ---- first contraction
    floatx16 acc[T2][T2];
    float xacc[T2];
    const ListBlock first = load_list_block<MODE == kKeySide>(csc_row, vals, gdb, beg, end);
    with_feature_map(fmap, [&](auto fm) {
        constexpr int FM = decltype(fm)::value;
        if constexpr (MODE == kQuerySide)
            bucket_first_contraction<D, T, T, true, false, kExtraSumB, FM, WIDE>(Vb, Kb, csc_row, vals, nullptr, beg, end, first, acc, xacc);
        else if constexpr (MODE == kKeySide)
            bucket_first_contraction<D, float, T, true, false, kExtraScaledSumB, FM, WIDE>(Gb, Qb, csc_row, vals, gdb, beg, end, first, acc, xacc);
        else
            bucket_first_contraction<D, T, float, true, true, kExtraNone, FM, WIDE>(Qb, Gb, csc_row, vals, nullptr, beg, end, first, acc, xacc);
    });

    // the extra row, complete in the lower half-wave and zero in the upper, so that one more MFMA step
    // (k = 0: the consumer's coefficient, k = 1: nothing) adds coefficient_i * extra to the output tile
    float extra[T2];
#pragma unroll
    for (int t = 0; t < T2; ++t) {
        const float full = xacc[t] + __shfl_xor(xacc[t], 32, kWave);
        extra[t] = half == 0 ? full : 0.0f;
    }

    // ---- second contraction, 32 consumers at a time.  The consumer's own weight Phi_hat[i, l] is left to the
    // reduce kernel, which is bound by memory, whereas vector instructions here are paid in matrix time.
    const long long pbase = slice * static_cast<long long>(nnz);
    for (int32_t tile = beg; tile < end; tile += 32) {
        float cop[4][QN];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e2 = 0; e2 < QN; ++e2)
                cop[b][e2] = MODE == kValueSide ? feature(cn[b][e2], fmap) : cn[b][e2];
        const float coef = half == 0 ? cfn : 0.0f;
        // next tile's operand rows, and the indices of the tile after it
        fetch_operand(row_next, cn, cfn);
        fetch_index(tile + 64, row_next);

        __builtin_amdgcn_sched_barrier(0);

        floatx16 pc[T2];
#pragma unroll
        for (int c = 0; c < T2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) pc[c][r] = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
#pragma unroll
            for (int t = 0; t < T2; ++t)
#pragma unroll
                for (int c = 0; c < T2; ++c)
                    pc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(cop[r / 4][T2 * (r % 4) + t], acc[t][c][r], pc[c], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (MODE != kValueSide) {
#pragma unroll
            for (int c = 0; c < T2; ++c)
                pc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(coef, extra[c], pc[c], 0, 0, 0);
        }

        // ---- stream out: register r of pc[c] is consumer tile + 8*(r/4) + 4*half + r%4, output column T2*li + c,
        // through a window over the tile's rows, which drops the rows past the end of the list.  One column tile
        // after the other, kept apart: merged into 8-byte stores, the two tiles' registers (never adjacent) would
        // have to be copied next to each other first.
        const __amdgpu_buffer_rsrc_t window = row_window(partial, pbase + tile, min(end - tile, 32), D);
        int lane_off = (4 * half * D + T2 * li) * 4;
        asm volatile("" : "+v"(lane_off));      // keeps the rows' constant offsets next to the stores, in their offset fields
#pragma unroll
        for (int c = 0; c < T2; ++c) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(pc[c][r]), window, lane_off + (8 * (r / 4) + (r % 4)) * D * 4 + 4 * c, 0, 0);
            asm volatile("" ::: "memory");
        }
    }
}

// One wavefront per (slice, row i) over the vectors streamed out for the row's entries, in ascending-l order:
// sum_l w_il u_il with w_il = Phi_hat[i, l].  WEIGHTED (gradients of Q and K): dst_i = phi'(x_i) * that sum, and the
// entry's term of dPhi, phi(x_i) . u_il, goes to dphi_part[slice][e] (CSR order).  Otherwise (gradient of V):
// dst_i = the sum.
template <int D, typename T, bool WEIGHTED>
__global__ __launch_bounds__(256) void backward_reduce_kernel(long long n, int H, int n_f, long long val_stride,
                                                              const int32_t* __restrict__ row_ptr, const float* __restrict__ phi_val,
                                                              const int32_t* __restrict__ csr_to_csc, int32_t nnz,
                                                              const float* __restrict__ partial, const T* __restrict__ src, int fmap,
                                                              long long bh_first, long long n_waves,
                                                              float* __restrict__ dst, float* __restrict__ dphi_part)
{
    constexpr int EPW = kWave / D;     // entries per wavefront step (1 at d = 64, 2 at d = 32)
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long i = wave - slice * n;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (bh % H) : 0;
    const float* vals = phi_val + plane * val_stride;
    const int lane = lane_id();
    const int sub = lane / D;
    const int c = lane % D;
    const float* slice_partial = partial + slice * static_cast<long long>(nnz) * D;
    const long long o = (bh * n + i) * D + c;
    float x = 0.0f, fx = 0.0f;
    if constexpr (WEIGHTED) { x = to_float(src[o]); fx = feature(x, fmap); }

    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    float acc = 0.0f;
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        const int32_t pos_reg = e < end ? csr_to_csc[e] : -1;
        const float w_reg = e < end ? vals[e] : 0.0f;
        const int cnt = min(kWave, end - chunk);
        // eight steps' loads are issued together; the shuffles are executed by every lane
        for (int t0 = 0; t0 < cnt; t0 += 8 * EPW) {
            float v[8], w[8];
            bool ok[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = t0 + u * EPW + sub;
                if constexpr (EPW == 1) {
                    // the entry is the same in every lane: a scalar broadcast, and a row address in scalar registers
                    // (the cross-lane unit is left to the dot products below); the load is unconditional
                    const int32_t pos = __builtin_amdgcn_readlane(pos_reg, t & (kWave - 1));
                    w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_reg), t & (kWave - 1)));
                    ok[u] = t < cnt && pos >= 0;
                    const float loaded = slice_partial[static_cast<long long>(max(pos, 0)) * D + c];
                    v[u] = ok[u] ? loaded : 0.0f;
                } else {
                    const int32_t pos = __shfl(pos_reg, t & (kWave - 1), kWave);
                    w[u] = __shfl(w_reg, t & (kWave - 1), kWave);
                    ok[u] = t < cnt && pos >= 0;
                    v[u] = ok[u] ? slice_partial[static_cast<long long>(pos) * D + c] : 0.0f;
                }
            }
            if constexpr (WEIGHTED) {
                float dot[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    acc = fmaf(w[u], v[u], acc);
                    dot[u] = fx * v[u];
                }
                // sum each dot[u] over the D lanes of its entry: three steps that halve the values a lane keeps
                // (exchanging the other half with the lane that keeps those), then plain butterfly steps
#pragma unroll
                for (int keep = 4, bit = D / 2; keep >= 1; keep >>= 1, bit >>= 1) {
                    const bool up = (c & bit) != 0;
#pragma unroll
                    for (int k = 0; k < keep; ++k) {
                        const float mine = up ? dot[k + keep] : dot[k];
                        const float theirs = up ? dot[k] : dot[k + keep];
                        dot[k] = mine + __shfl_xor(theirs, bit, kWave);
                    }
                }
#pragma unroll
                for (int bit = D / 16; bit >= 1; bit >>= 1) dot[0] += __shfl_xor(dot[0], bit, kWave);
                // this lane now holds step u = c / (D / 8) of the eight
                const int t = t0 + (c / (D / 8)) * EPW + sub;
                if ((c & (D / 8 - 1)) == 0 && t < cnt) dphi_part[slice * static_cast<long long>(nnz) + chunk + t] = dot[0];
            } else {
#pragma unroll
                for (int u = 0; u < 8; ++u) acc = fmaf(w[u], v[u], acc);
            }
        }
    }
    if constexpr (EPW == 2) acc += __shfl_xor(acc, 32, kWave);
    if (sub == 0) {
        if constexpr (WEIGHTED) acc *= feature_grad(x, fmap);
        dst[o] = acc;
    }
}

// The same at d = 64 in the layout of the gather kernel: 16 lanes share an entry (each holds four columns, one 16-byte
// load), so a wavefront step covers four entries and the per-entry dot product of dPhi is a sum over the 16 lanes of a
// row of the wavefront, formed with four row rotations on the vector ALU (no trips through the LDS crossbar, which the
// one-lane-per-column layout needs ten of per eight entries: with them the kernel ran at 3.8 TB/s against the 5.4 TB/s
// of its sibling without dot products).
template <typename T, bool WEIGHTED>
__global__ __launch_bounds__(256) void backward_reduce64_kernel(long long n, int H, int n_f, long long val_stride,
                                                                const int32_t* __restrict__ row_ptr, const float* __restrict__ phi_val,
                                                                const int32_t* __restrict__ csr_to_csc, int32_t nnz,
                                                                const float* __restrict__ partial, const T* __restrict__ src, int fmap,
                                                                long long bh_first, long long n_waves,
                                                                float* __restrict__ dst, float* __restrict__ dphi_part)
{
    constexpr int D = 64, LPR = D / 4, GROUPS = kWave / LPR, U = 8;      // U loads of a lane in flight: 32 entries
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long i = wave - slice * n;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (bh % H) : 0;
    const float* vals = phi_val + plane * val_stride;
    const int lane = lane_id();
    const int grp = lane / LPR;
    const int cl = lane % LPR;
    const float4* slice_partial = reinterpret_cast<const float4*>(partial + slice * static_cast<long long>(nnz) * D);
    const long long o = (bh * n + i) * D + 4 * cl;
    float xs[4] = {0.0f, 0.0f, 0.0f, 0.0f}, fx[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (WEIGHTED) {
        load_run<T, 4>(src + o, xs);
#pragma unroll
        for (int k = 0; k < 4; ++k) fx[k] = feature(xs[k], fmap);
    }

    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        const int32_t pos_reg = e < end ? csr_to_csc[e] : -1;
        const float w_reg = e < end ? vals[e] : 0.0f;
        const int cnt = min(kWave, end - chunk);
        for (int t0 = 0; t0 < cnt; t0 += GROUPS * U) {
            float4 v[U];
            float w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0 + GROUPS * u + grp;      // this group's entry of the step; the loads are unconditional
                const int32_t pos = __shfl(pos_reg, t & (kWave - 1), kWave);
                const float wt = __shfl(w_reg, t & (kWave - 1), kWave);
                const bool ok = t < cnt && pos >= 0;
                const float4 loaded = slice_partial[static_cast<long long>(max(pos, 0)) * LPR + cl];
                v[u] = ok ? loaded : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                w[u] = ok ? wt : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                acc[0] = fmaf(w[u], v[u].x, acc[0]);
                acc[1] = fmaf(w[u], v[u].y, acc[1]);
                acc[2] = fmaf(w[u], v[u].z, acc[2]);
                acc[3] = fmaf(w[u], v[u].w, acc[3]);
                if constexpr (WEIGHTED) {
                    float dot = fmaf(fx[0], v[u].x, fmaf(fx[1], v[u].y, fmaf(fx[2], v[u].z, fx[3] * v[u].w)));
                    dot = row_sum16(dot);
                    const int t = t0 + GROUPS * u + grp;
                    if (cl == 0 && t < cnt) dphi_part[slice * static_cast<long long>(nnz) + chunk + t] = dot;
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        acc[k] += __shfl_xor(acc[k], 16, kWave);
        acc[k] += __shfl_xor(acc[k], 32, kWave);
    }
    if (grp == 0) {
        if constexpr (WEIGHTED) {
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] *= feature_grad(xs[k], fmap);
        }
        *reinterpret_cast<float4*>(dst + o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
}

// dphi_val[h][e] (+)= sum over the slices of this chunk that use plane h of the two per-entry terms; entries past the
// end of the rows (nnz may be an upper bound: the rows end at row_ptr[n]) receive 0.  A workgroup
// covers 32 consecutive entries; its 8 groups of 32 threads take the slices s = g, g + 8, ... in order and the groups'
// sums are added in group order, so the result has a fixed summation order for a given chunking.
__global__ __launch_bounds__(256) void dphi_accumulate_kernel(long long nnz, int n_f, int H, long long bh_first, long long n_slices,
                                                              const float* __restrict__ d_query, const float* __restrict__ d_key,
                                                              long long val_stride, int first_chunk, const int32_t* __restrict__ row_ptr,
                                                              long long n, float* __restrict__ dphi_val)
{
    constexpr int kEntries = 32, kGroups = 8;
    __shared__ float part[kGroups][kEntries];
    const int lane = threadIdx.x % kEntries, group = threadIdx.x / kEntries;
    const long long e = static_cast<long long>(blockIdx.x) * kEntries + lane;
    const int h = blockIdx.y;
    float acc = 0.0f;
    const bool live = e < nnz && e < row_ptr[n];
    if (live) {
        for (long long s = group; s < n_slices; s += kGroups) {
            const long long bh = bh_first + s;
            if (n_f > 1 && bh % H != h) continue;
            acc += d_query[s * nnz + e];
            if (d_key != nullptr) acc += d_key[s * nnz + e];
        }
    }
    part[group][lane] = acc;
    __syncthreads();
    if (group == 0 && e < nnz) {
        float total = (first_chunk || !live) ? 0.0f : dphi_val[h * val_stride + e];
#pragma unroll
        for (int g = 0; g < kGroups; ++g) total += part[g][lane];
        dphi_val[h * val_stride + e] = total;
    }
}

grf_status launch_backward_seed(int32_t d, const float* out, const float* den, const float* d_out, long long first_row,
                                long long n_rows, float* G, float* gd, hipStream_t stream)
{
    if (n_rows <= 0) return GRF_OK;
    if (d == 64) {
        hipLaunchKernelGGL((backward_seed_kernel<64>), dim3(blocks_for(n_rows, 4)), dim3(256), 0, stream, out, den, d_out, first_row, n_rows, G, gd);
    } else {
        hipLaunchKernelGGL((backward_seed_kernel<32>), dim3(blocks_for((n_rows + 1) / 2, 4)), dim3(256), 0, stream, out, den, d_out, first_row, n_rows, G, gd);
    }
    GRF_LAUNCH_CHECK("backward_seed_kernel");
    return GRF_OK;
}

grf_status launch_dphi_accumulate(int64_t nnz, int32_t n_f, int64_t H, int64_t bh_first, int64_t n_slices,
                                  const float* term_a, const float* term_b, const grf_phi* phi, float* dphi_val,
                                  hipStream_t stream)
{
    const int64_t val_stride = phi->capacity;
    if (dphi_val == nullptr || nnz <= 0) return GRF_OK;
    hipLaunchKernelGGL(dphi_accumulate_kernel, dim3(blocks_for(nnz, 32), static_cast<unsigned>(n_f)), dim3(256), 0, stream,
                       static_cast<long long>(nnz), static_cast<int>(n_f), static_cast<int>(H), static_cast<long long>(bh_first),
                       static_cast<long long>(n_slices), term_a, term_b, static_cast<long long>(val_stride), bh_first == 0 ? 1 : 0,
                       static_cast<const int32_t*>(phi->row_ptr), static_cast<long long>(phi->n), dphi_val);
    GRF_LAUNCH_CHECK("dphi_accumulate_kernel");
    return GRF_OK;
}

namespace {

struct BackwardScratch {
    float* G;          // [chunk][n][d]
    float* gd;         // [chunk][n]
    float* partial;    // [chunk][nnz][d]
    float* d_query;    // [chunk][nnz], CSR order: phi(q_i) . U_il
    float* d_key;      // [chunk][nnz], CSR order: phi(k_i) . R_il
    size_t bytes;
};

BackwardScratch carve_backward(unsigned char* ws, int64_t slices, int64_t n, int32_t d, int64_t nnz)
{
    BackwardScratch b;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = ws ? ws + off : nullptr; off += align_up(bytes); return reinterpret_cast<float*>(p); };
    const size_t entries = static_cast<size_t>(nnz > 0 ? nnz : 1), rows = static_cast<size_t>(n > 0 ? n : 1), sl = static_cast<size_t>(slices > 0 ? slices : 1);
    b.G = take(sizeof(float) * sl * rows * d);
    b.gd = take(sizeof(float) * sl * rows);
    b.partial = take(sizeof(float) * sl * entries * d);
    b.d_query = take(sizeof(float) * sl * entries);
    b.d_key = take(sizeof(float) * sl * entries);
    b.bytes = off;
    return b;
}

template <int D, typename T>
grf_status launch_backward_chunk(const void* Qv, const void* Kv, const void* Vv, int64_t n, int64_t H, int32_t n_f,
                                 const grf_phi* phi, int64_t nnz, const Transposed& t, const BackwardScratch& b, int fmap,
                                 int64_t bh_first, int64_t n_slices, const float* out, const float* den, const float* d_out,
                                 float* dQ, float* dK, float* dV, float* dphi_val, hipStream_t stream)
{
    const T* Q = static_cast<const T*>(Qv);
    const T* K = static_cast<const T*>(Kv);
    const T* V = static_cast<const T*>(Vv);
    const long long waves = static_cast<long long>(n_slices) * n;
    if (waves == 0) return GRF_OK;
    if (D == 64 && static_cast<long long>(n_slices) * t.item_capacity >= 2147483647ll)
        return fail(GRF_EUNSUPPORTED, "slices * nnz / 8 = %lld * %lld must be < 2^31", (long long)n_slices, t.item_capacity);
    if (grf_status st = launch_backward_seed(D, out, den, d_out, static_cast<long long>(bh_first) * n, waves, b.G, b.gd, stream)) return st;

    const dim3 bucket_grid(blocks_for(waves, 1)), reduce_grid(blocks_for(waves, 4));
    const int32_t* col_ptr = t.col_ptr;
    const int32_t* s_row = t.s_row;
    const float* s_val = t.s_val;
    const int32_t* csr_to_csc = t.csr_to_csc;
    const int32_t* row_ptr = phi->row_ptr;
    const float* partial = b.partial;

    const float* phi_val = phi->val;
    const long long val_stride = phi->capacity;
    const bool wide = wide_offsets(n, D);
    // eight slices' Q, K, V and G within a quarter of the 256 MB Infinity Cache: see the kernel
    const int spread = 8ll * n * D * (3 * static_cast<long long>(sizeof(T)) + 4) <= (64ll << 20) ? 1 : 0;
    auto bucket_pass = [&](auto mode) {
        auto launch = [&](auto w) {
            if constexpr (D == 64) {      // on the bf16 matrix cores: short lists several buckets per wavefront, the others one each
                auto gram = gram_bucket_kernel<T, decltype(mode)::value, decltype(w)::value>;
                hipLaunchKernelGGL(gram, dim3(resident_wave_grid(reinterpret_cast<const void*>(gram), static_cast<long long>(n_slices) * t.item_capacity)),
                                   dim3(kWave), 0, stream,
                                   Q, K, V, static_cast<const float*>(b.G), static_cast<const float*>(b.gd), static_cast<long long>(n),
                                   static_cast<int>(H), static_cast<int>(n_f), static_cast<const int2*>(t.items),
                                   static_cast<const int32_t*>(t.plan_counts), s_row, static_cast<const int32_t*>(t.span), s_val, fmap,
                                   static_cast<long long>(bh_first), static_cast<uint32_t>(n_slices), static_cast<int32_t>(nnz), spread,
                                   b.partial, static_cast<float*>(nullptr));
                auto go = [&](auto kernel, bool listed) {
                    const dim3 grid = listed ? dim3(resident_wave_grid(reinterpret_cast<const void*>(kernel), waves)) : bucket_grid;
                    hipLaunchKernelGGL(kernel, grid, dim3(kWave), 0, stream, Q, K, V,
                                       static_cast<const float*>(b.G), static_cast<const float*>(b.gd), static_cast<long long>(n),
                                       static_cast<int>(H), static_cast<int>(n_f), col_ptr, s_row, s_val, fmap,
                                       static_cast<long long>(bh_first), waves, static_cast<int32_t>(nnz), spread,
                                       static_cast<const int32_t*>(t.long_list), static_cast<const int32_t*>(t.plan_counts), b.partial);
                };
                if (few_long_lists(n, nnz)) go(backward_bucket_split_kernel<T, decltype(mode)::value, decltype(w)::value, true>, true);
                else go(backward_bucket_split_kernel<T, decltype(mode)::value, decltype(w)::value, false>, false);
            } else {
                hipLaunchKernelGGL((backward_bucket_kernel<D, T, decltype(mode)::value, decltype(w)::value>), bucket_grid, dim3(kWave), 0, stream, Q, K, V,
                                   static_cast<const float*>(b.G), static_cast<const float*>(b.gd), static_cast<long long>(n),
                                   static_cast<int>(H), static_cast<int>(n_f), col_ptr, s_row, s_val, fmap,
                                   static_cast<long long>(bh_first), waves, static_cast<int32_t>(nnz), spread, b.partial);
            }
        };
        if (wide) launch(std::true_type{}); else launch(std::false_type{});
    };
    auto reduce_pass = [&](auto weighted, const T* src, float* dst, float* dphi_part) {
        if constexpr (D == 64) {
            hipLaunchKernelGGL((backward_reduce64_kernel<T, decltype(weighted)::value>), reduce_grid, dim3(256), 0, stream,
                               static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f), val_stride, row_ptr, phi_val,
                               csr_to_csc, static_cast<int32_t>(nnz), partial, src, fmap, static_cast<long long>(bh_first), waves,
                               dst, dphi_part);
            return;
        }
        hipLaunchKernelGGL((backward_reduce_kernel<D, T, decltype(weighted)::value>), reduce_grid, dim3(256), 0, stream,
                           static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f), val_stride, row_ptr, phi_val,
                           csr_to_csc, static_cast<int32_t>(nnz), partial, src, fmap, static_cast<long long>(bh_first), waves,
                           dst, dphi_part);
    };
    bucket_pass(std::integral_constant<int, kQuerySide>{});
    GRF_LAUNCH_CHECK("backward_bucket_kernel<query side>");
    reduce_pass(std::true_type{}, Q, dQ, b.d_query);
    GRF_LAUNCH_CHECK("backward_reduce_kernel<dQ>");
    bucket_pass(std::integral_constant<int, kKeySide>{});
    GRF_LAUNCH_CHECK("backward_bucket_kernel<key side>");
    reduce_pass(std::true_type{}, K, dK, b.d_key);
    GRF_LAUNCH_CHECK("backward_reduce_kernel<dK>");
    bucket_pass(std::integral_constant<int, kValueSide>{});
    GRF_LAUNCH_CHECK("backward_bucket_kernel<value side>");
    reduce_pass(std::false_type{}, V, dV, static_cast<float*>(nullptr));
    GRF_LAUNCH_CHECK("backward_reduce_kernel<dV>");

    if (grf_status st = launch_dphi_accumulate(nnz, n_f, H, bh_first, n_slices, b.d_query, b.d_key, phi, dphi_val, stream)) return st;
    return GRF_OK;
}

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" size_t grf_attention_backward_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk)
{
    if (B < 0 || H < 0 || n < 0 || nnz < 0 || n_f < 1 || (d != 32 && d != 64)) return 0;
    int64_t slices = B * H;
    if (bh_chunk > 0 && bh_chunk < slices) slices = bh_chunk;
    return carve_transposed(nullptr, n, nnz, n_f).bytes + carve_backward(nullptr, slices, n, d, nnz).bytes;
}

namespace {

grf_status backward_chunks(const void* Q, const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                           const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map, const float* out, const float* den,
                           const float* d_out, int64_t step, const Transposed& t, unsigned char* rest, hipStream_t stream,
                           float* dQ, float* dK, float* dV, float* dphi_val)
{
    const int64_t slices = B * H;
    const BackwardScratch b = carve_backward(rest, step, n, d, nnz);
    for (int64_t first = 0; first < slices; first += step) {
        const int64_t count = (slices - first < step) ? (slices - first) : step;
        grf_status st = GRF_OK;
        GRF_DISPATCH(d, dtype, (st = launch_backward_chunk<D_, T_>(Q, K, V, n, H, n_f, phi, nnz, t, b, feature_map, first, count,
                                                                   out, den, d_out, dQ, dK, dV, dphi_val, stream)));
        if (st != GRF_OK) return st;
    }
    return GRF_OK;
}

// Argument checks shared by the two forms; *done is set when there is nothing to launch.
grf_status backward_checks(const void* Q, const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                           const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map, const float* out, const float* den,
                           const float* d_out, float* dQ, float* dK, float* dV)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr || den == nullptr || d_out == nullptr))
        return fail(GRF_EINVAL, "Q / out / den / d_out is NULL");
    if (B * H * n > 0 && (dQ == nullptr || dK == nullptr || dV == nullptr)) return fail(GRF_EINVAL, "dQ / dK / dV is NULL");
    return GRF_OK;
}

// no slices: the gradient with respect to Phi_hat is zero
grf_status zero_dphi(const grf_phi* phi, int64_t nnz, int32_t n_f, float* dphi_val, hipStream_t stream)
{
    if (dphi_val != nullptr && nnz > 0)
        for (int32_t h = 0; h < n_f; ++h)
            if (grf_status st = fill_i32(reinterpret_cast<int32_t*>(dphi_val + static_cast<int64_t>(h) * phi->capacity), nnz, 0, stream)) return st;
    return GRF_OK;
}

}  // namespace

extern "C" grf_status grf_masked_linear_attention_backward(const void* Q, const void* K, const void* V, int32_t dtype,
                                                           int64_t B, int64_t H, int64_t n, int32_t d,
                                                           const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                           const float* out, const float* den, const float* d_out,
                                                           int32_t bh_chunk,
                                                           void* workspace, size_t workspace_bytes, void* hip_stream,
                                                           float* dQ, float* dK, float* dV, float* dphi_val)
{
    if (grf_status st = backward_checks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, out, den, d_out, dQ, dK, dV)) return st;
    if (grf_status st = check_workspace(workspace, workspace_bytes, grf_attention_backward_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B * H * n == 0) return zero_dphi(phi, nnz, n_f, dphi_val, stream);
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const Transposed t = carve_transposed(ws, n, nnz, n_f);
    if (grf_status st = transpose(phi, nnz, n_f, t, stream)) return st;
    return backward_chunks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, out, den, d_out, step, t, ws + t.bytes, stream,
                           dQ, dK, dV, dphi_val);
}

extern "C" grf_status grf_masked_linear_attention_backward_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
                                                                    int64_t B, int64_t H, int64_t n, int32_t d,
                                                                    const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                                    const float* out, const float* den, const float* d_out,
                                                                    int32_t bh_chunk, const void* prepared, size_t prepared_bytes,
                                                                    void* workspace, size_t workspace_bytes, void* hip_stream,
                                                                    float* dQ, float* dK, float* dV, float* dphi_val)
{
    if (grf_status st = backward_checks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, out, den, d_out, dQ, dK, dV)) return st;
    Transposed t;
    if (grf_status st = prepared_lists(prepared, prepared_bytes, n, nnz, n_f, &t)) return st;
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    if (grf_status st = check_workspace(workspace, workspace_bytes, carve_backward(nullptr, step, n, d, nnz).bytes)) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (B * H * n == 0) return zero_dphi(phi, nnz, n_f, dphi_val, stream);
    return backward_chunks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, out, den, d_out, step, t,
                           static_cast<unsigned char*>(workspace), stream, dQ, dK, dV, dphi_val);
}
