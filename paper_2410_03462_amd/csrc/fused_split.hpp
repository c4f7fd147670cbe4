// Bucket-fused evaluation (Eq. 7; Alg. 1 steps 3-5) at d = 64 on the bf16 matrix cores with fp32-grade products
// (fp32 inputs; bf16 inputs under a feature map whose values are not bf16 numbers).
//
// v_mfma_f32_32x32x2_f32 shares the vector ALU and delivers 157 TFLOP/s; v_mfma_f32_32x32x16_bf16 runs beside
// the vector ALU at sixteen times that rate.  An fp32 number is exactly the sum of three bf16 numbers
// (h = nearest bf16 of x, m = nearest bf16 of x - h, l = nearest bf16 of x - h - m), products of bf16 numbers
// are exact in fp32 and the matrix cores accumulate in fp32, so
//     a b  =  a_h b_h + (a_h b_m + a_m b_h) + (a_h b_l + a_l b_h + a_m b_m)  +  O(2^-23 |a b|)
// is an fp32 product from six bf16 MFMAs: for a depth of 16, 6 x 34 cycles against 8 x 60 of the fp32 instruction.
// Both contractions of a bucket are done this way; the vector ALU does the splitting.
//
// Index convention as in the bf16-input kernel: MFMA row/column x of tile t stands for feature / value column
// 2x + t (a lane's two tiles are the two floats of one 8-byte load).  Lane L = 32 g + f; in every operand the
// lanes of group g carry depth slots (g, 0..7) of the instruction, two bf16 per register.
#pragma once

#include "split_common.hpp"

namespace grf {

// First contraction of a bucket at d = 64 with three-piece operands: acc[a][c] = A^T B over the column list
// [beg, end) with A = Phi_hat[j,l] phi(k_j), B = v_j (MFMA row/column x of tile t stands for element 2x + t), and
// zacc[a] = this lane's share of z_l = A^T 1: the sum over lanes f and 32 + f is z_l[2f + a].  16 members of the
// list per step: lane (g, f) takes members 8 g + 0..7 of the step from the list block with ds_bpermute and loads
// elements 2f, 2f + 1 of their rows of K and V.
template <typename T, bool WIDE>
__device__ __forceinline__ void bucket_first_contraction_split(const T* __restrict__ Kb, const T* __restrict__ Vb,
                                                               const int32_t* __restrict__ csc_row, const float* __restrict__ vals,
                                                               int fmap, int32_t beg, int32_t end,
                                                               floatx16 (&acc)[2][2], float (&zacc)[2])
{
    const int lane = lane_id();
    const int g = lane >> 5;
    const int f = lane & 31;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        zacc[a] = 0.0f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
    }
    if (beg >= end) return;      // an empty list: zeros, and no row is read
    struct Members { typename RawPair<T>::type k[8], v[8]; float w[8]; };
    auto fetch_members = [&](int32_t jv, float gv, int first, Members& m) {
        int addr = 4 * ((first + 8 * g) & (kWave - 1));
        asm volatile("" : "+v"(addr));      // one register, the members' offsets as literals
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t row = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr + 4 * j, jv));
            m.w[j] = __int_as_float(__builtin_amdgcn_ds_bpermute(addr + 4 * j, __float_as_int(gv)));
            m.k[j] = load_pair<T, WIDE>(Kb, row, f);
            m.v[j] = load_pair<T, WIDE>(Vb, row, f);
        }
    };
    auto contract_members = [&](const Members& m) {
        uint32_t a_p[2][3][4], b_p[2][3][4];      // [tile][piece][register]
        with_feature_map(fmap, [&](auto fm) {
            constexpr int FM = decltype(fm)::value;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float2 k0 = widen(m.k[2 * p]), k1 = widen(m.k[2 * p + 1]);
                const float x0 = m.w[2 * p] * feature_ct<FM>(k0.x), x1 = m.w[2 * p + 1] * feature_ct<FM>(k1.x);
                const float y0 = m.w[2 * p] * feature_ct<FM>(k0.y), y1 = m.w[2 * p + 1] * feature_ct<FM>(k1.y);
                zacc[0] += x0 + x1;
                zacc[1] += y0 + y1;
                split3_bf16(x0, x1, a_p[0][0][p], a_p[0][1][p], a_p[0][2][p]);
                split3_bf16(y0, y1, a_p[1][0][p], a_p[1][1][p], a_p[1][2][p]);
            }
        });
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const float2 v0 = widen(m.v[2 * p]), v1 = widen(m.v[2 * p + 1]);
            split3_bf16(v0.x, v1.x, b_p[0][0][p], b_p[0][1][p], b_p[0][2][p]);
            split3_bf16(v0.y, v1.y, b_p[1][0][p], b_p[1][1][p], b_p[1][2][p]);
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c) mfma_split3(a_p[a], b_p[c], acc[a][c]);
    };

    walk_column_list<Members, false>(csc_row, vals, nullptr, beg, end,
                                     [&](int32_t jv, float gv, float, int first, Members& m) { fetch_members(jv, gv, first, m); },
                                     [&](const Members& m, float, float, int) { contract_members(m); });
}

// One wavefront per (slice, bucket l), one wavefront per workgroup; structure as fused_bucket_bf16_kernel:
// 16 members of the column list per step of the first contraction (lane (g, f) takes members 8 g + 0..7 and
// loads floats 2f, 2f + 1 of their rows of K and V), 32 consumers per step of the second, whose B operand is
// the accumulators' registers 8 h + 0..7 split into pieces once per bucket.  z_l is summed on the vector ALU
// beside the first contraction and handed to the lanes in the order of their depth slots with ds_bpermute; the
// partial denominator phi(q) . z_l is 32 fused multiply-adds per lane and tile.
template <typename T, bool WIDE, bool LISTED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void fused_bucket_split_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, long long n, int H, int n_f,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row, const float* __restrict__ csc_val, int fmap,
    long long bh_first, long long n_waves, int32_t nnz, int spread_xcds, const int32_t* __restrict__ long_list,
    const int32_t* __restrict__ plan_counts, float* __restrict__ partial, float* __restrict__ pden)
{
    constexpr int D = 64;
    for_each_long_bucket<LISTED>(n, n_waves, spread_xcds, long_list, plan_counts, [&](uint32_t slice32, uint32_t l32) {
    const long long slice = slice32;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (static_cast<uint32_t>(bh) % static_cast<uint32_t>(H)) : 0u;
    const T* Qb = Q + bh * n * D;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;
    const float* vals = csc_val + plane * nnz;

    const int lane = lane_id();
    const int g = lane >> 5;
    const int f = lane & 31;

    const int32_t beg = __builtin_amdgcn_readfirstlane(col_ptr[l32]);
    const int32_t end = __builtin_amdgcn_readfirstlane(col_ptr[l32 + 1]);
    if (end - beg <= kGramMaxList) return;      // short lists (and empty ones) belong to gram_bucket_kernel

    // consumer f's q at the features of depth slots (g, .): elements 2 rho, 2 rho + 1 for rho = 8 hr + 4 g + 0..3
    auto fetch_q = [&](int32_t row, float (&qw)[4][8]) {
#pragma unroll
        for (int hr = 0; hr < 4; ++hr) load_eight<T, WIDE>(Qb, static_cast<uint32_t>(row), 2 * (8 * hr + 4 * g), qw[hr]);
    };
    auto fetch_index = [&](int32_t tile, int32_t& row) { row = csc_row[min(tile + f, end - 1)]; };

    // the first two consumer tiles' indices and the first tile's rows of Q go out before the first contraction
    int32_t qrow_cur, qrow_next;
    fetch_index(beg, qrow_cur);
    fetch_index(beg + 32, qrow_next);
    float qn[4][8];
    fetch_q(qrow_cur, qn);

    // ---- S_l = A^T V_l, z_l = A^T 1
    floatx16 acc[2][2];
    float zacc[2];
    bucket_first_contraction_split<T, WIDE>(Kb, Vb, csc_row, vals, fmap, beg, end, acc, zacc);

    // ---- z_l at the features of this lane's depth slots: lane rho of either group holds z[2 rho + a]
    float zs[2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const float zfull = zacc[a] + __shfl_xor(zacc[a], 32, kWave);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            zs[a][r] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (8 * (r / 4) + 4 * g + (r % 4)), __float_as_int(zfull)));
    }

    // ---- the accumulators in pieces, in the registers' own order: [a][c][h] holds registers 8 h + 0..7
    uint32_t s_p[2][2][2][3][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    split3_bf16(acc[a][c][8 * h + 2 * p], acc[a][c][8 * h + 2 * p + 1], s_p[a][c][h][0][p], s_p[a][c][h][1][p], s_p[a][c][h][2][p]);

    // ---- P_l = phi(Q_l) S_l and pden_l = phi(Q_l) z_l, 32 consumers at a time
    const long long pbase = slice * nnz;
    for (int32_t tile = beg; tile < end; tile += 32) {
        // phi(q) of this tile, register 8 h + j of depth slot (g, j): feature 2 (8 (2 h + j / 4) + 4 g + j % 4) + a
        float fq[2][16];
        with_feature_map(fmap, [&](auto fm) {
            constexpr int FM = decltype(fm)::value;
#pragma unroll
            for (int hr = 0; hr < 4; ++hr)
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int a = 0; a < 2; ++a) fq[a][4 * hr + k] = feature_ct<FM>(qn[hr][2 * k + a]);
        });
        // next tile's rows of Q, and the indices of the tile after it
        fetch_q(qrow_next, qn);
        fetch_index(tile + 64, qrow_next);

        float dl = 0.0f;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int r = 0; r < 16; ++r) dl = fmaf(fq[a][r], zs[a][r], dl);
        dl += __shfl_xor(dl, 32, kWave);
        if (g == 0 && tile + f < end) pden[pbase + tile + f] = dl;

        floatx16 pc[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) { pc[0][r] = 0.0f; pc[1][r] = 0.0f; }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t q_p[3][4];
#pragma unroll
                for (int p = 0; p < 4; ++p) split3_bf16(fq[a][8 * h + 2 * p], fq[a][8 * h + 2 * p + 1], q_p[0][p], q_p[1][p], q_p[2][p]);
#pragma unroll
                for (int c = 0; c < 2; ++c) mfma_split3(q_p, s_p[a][c][h], pc[c]);
            }

        store_consumer_tile(partial, pbase + tile, min(end - tile, 32), g, f, pc[0], pc[1]);
    }
    });
}

}  // namespace grf
