// The three bucket passes of the backward pass (gradients of Eq. 7) at d = 64 on the bf16 matrix cores: fp32
// operands enter as three bf16 pieces and every product is six bf16 MFMAs (see fused_split.hpp), which takes well
// under half the matrix time of v_mfma_f32_32x32x2_f32 and runs beside the vector ALU instead of on it.
//
//   pass           first contraction ACC = A^T B            second contraction, per consumer i     streams out
//   kQuerySide     A = V,        B = w phi(K), x = sum B     U_i = g_i ACC + gd_i x                 U_i
//   kKeySide       A = G,        B = w phi(Q), x = sum gd B  R_i = v_i ACC + x                      R_i
//   kValueSide     A = w phi(Q), B = G                       X_i = phi(k_i) ACC                     X_i
//
// Index convention as in the forward kernels: MFMA row/column x of tile t stands for element 2x + t of a row.
// Lane L = 32 g + f; in every operand the lanes of group g carry depth slots (g, 0..7), two bf16 per register.
#pragma once

#include "split_common.hpp"

namespace grf {

// One wavefront per (slice, bucket l), one wavefront per workgroup; every global load is unconditional (members
// past the end of the column list re-read its last entry with weight 0).  16 members of the list per step of the
// first contraction (lane (g, f) takes members 8 g + 0..7 and loads elements 2f, 2f + 1 of their two rows), 32
// consumers per step of the second, whose B operand is the accumulators' registers 8 h + 0..7 split into pieces
// once per bucket.  The extra row x is summed on the vector ALU beside the first contraction; its column 2f + c
// ends up in lane f, which is the column that lane's output registers hold, so the output tile starts from
// coefficient * x (the coefficients of the registers' consumers come over with ds_bpermute) instead of from zero.
template <typename T, int MODE, bool WIDE, bool LISTED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void backward_bucket_split_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const float* __restrict__ G, const float* __restrict__ gd,
    long long n, int H, int n_f, const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row,
    const float* __restrict__ csc_val, int fmap, long long bh_first, long long n_waves, int32_t nnz, int spread_xcds,
    const int32_t* __restrict__ long_list, const int32_t* __restrict__ plan_counts, float* __restrict__ partial)
{
    constexpr int D = 64;
    // pieces per operand: fp32-grade products for fp32 inputs; with bf16 inputs (bar 2e-2) two pieces, three products
    constexpr int NP = sizeof(T) == 2 ? 2 : 3;
    for_each_long_bucket<LISTED>(n, n_waves, spread_xcds, long_list, plan_counts, [&](uint32_t slice32, uint32_t l32) {
    const long long slice = slice32;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (static_cast<uint32_t>(bh) % static_cast<uint32_t>(H)) : 0u;
    const T* Qb = Q + bh * n * D;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;
    const float* Gb = G + slice * n * D;
    const float* gdb = gd + slice * n;
    const float* vals = csc_val + plane * nnz;

    const int lane = lane_id();
    const int g = lane >> 5;
    const int f = lane & 31;

    const int32_t beg = __builtin_amdgcn_readfirstlane(col_ptr[l32]);
    const int32_t end = __builtin_amdgcn_readfirstlane(col_ptr[l32 + 1]);
    if (end - beg <= kGramMaxList) return;      // short lists (and empty ones) belong to gram_bucket_kernel

    // consumer f's operand of the second contraction at the elements of depth slots (g, .): elements 2 rho,
    // 2 rho + 1 for rho = 8 hr + 4 g + 0..3; and its coefficient of the extra row
    auto fetch_operand = [&](int32_t row, float (&cw)[4][8], float& cf) {
        const uint32_t r = static_cast<uint32_t>(row);
#pragma unroll
        for (int hr = 0; hr < 4; ++hr) {
            const int elem = 2 * (8 * hr + 4 * g);
            if constexpr (MODE == kQuerySide) load_eight<float, WIDE>(Gb, r, elem, cw[hr]);
            if constexpr (MODE == kKeySide) load_eight<T, WIDE>(Vb, r, elem, cw[hr]);
            if constexpr (MODE == kValueSide) load_eight<T, WIDE>(Kb, r, elem, cw[hr]);
        }
        if constexpr (MODE == kQuerySide) cf = gdb[row];
    };
    auto fetch_index = [&](int32_t tile, int32_t& row) { row = csc_row[min(tile + f, end - 1)]; };

    // the first two consumer tiles' indices go out before the first contraction
    int32_t row_cur, row_next;
    fetch_index(beg, row_cur);
    fetch_index(beg + 32, row_next);

    // ---- first contraction
    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
    float xacc[2] = {0.0f, 0.0f};

    // the rows of a step's members as loaded; their weights (and, on the key side, their coefficients of the extra
    // row) are taken from the list block only when the step is contracted
    typedef typename std::conditional<MODE == kKeySide, float, T>::type TA;
    typedef typename std::conditional<MODE == kValueSide, float, T>::type TB;
    struct Members { typename RawPair<TA>::type a[8]; typename RawPair<TB>::type b[8]; };
    // members first + 8 g + 0..7 of the 64 entries held one per lane
    auto member_address = [&](int first) {
        int addr = 4 * ((first + 8 * g) & (kWave - 1));
        asm volatile("" : "+v"(addr));      // one register, the members' offsets as literals
        return addr;
    };
    auto fetch_members = [&](int32_t jv, int first, Members& m) {
        const int addr = member_address(first);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t row = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr + 4 * j, jv));
            if constexpr (MODE == kQuerySide) { m.a[j] = load_pair<T, WIDE>(Vb, row, f); m.b[j] = load_pair<T, WIDE>(Kb, row, f); }
            if constexpr (MODE == kKeySide) { m.a[j] = load_pair<float, WIDE>(Gb, row, f); m.b[j] = load_pair<T, WIDE>(Qb, row, f); }
            if constexpr (MODE == kValueSide) { m.a[j] = load_pair<T, WIDE>(Qb, row, f); m.b[j] = load_pair<float, WIDE>(Gb, row, f); }
        }
    };
    auto contract_members = [&](const Members& m, float gv, float ev, int first) {
        const int addr = member_address(first);
        float w[8], e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            w[j] = __int_as_float(__builtin_amdgcn_ds_bpermute(addr + 4 * j, __float_as_int(gv)));
            if constexpr (MODE == kKeySide) e[j] = __int_as_float(__builtin_amdgcn_ds_bpermute(addr + 4 * j, __float_as_int(ev)));
        }
        uint32_t a_p[2][NP][4], b_p[2][NP][4];      // [tile][piece][register]
        with_feature_map(fmap, [&](auto fm) {
            constexpr int FM = decltype(fm)::value;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                float2 a0 = widen(m.a[2 * p]), a1 = widen(m.a[2 * p + 1]), b0 = widen(m.b[2 * p]), b1 = widen(m.b[2 * p + 1]);
                const float w0 = w[2 * p], w1 = w[2 * p + 1];
                if constexpr (MODE == kValueSide) {
                    a0 = make_float2(w0 * feature_ct<FM>(a0.x), w0 * feature_ct<FM>(a0.y));
                    a1 = make_float2(w1 * feature_ct<FM>(a1.x), w1 * feature_ct<FM>(a1.y));
                } else {
                    b0 = make_float2(w0 * feature_ct<FM>(b0.x), w0 * feature_ct<FM>(b0.y));
                    b1 = make_float2(w1 * feature_ct<FM>(b1.x), w1 * feature_ct<FM>(b1.y));
                }
                if constexpr (MODE == kQuerySide) { xacc[0] += b0.x + b1.x; xacc[1] += b0.y + b1.y; }
                if constexpr (MODE == kKeySide) {
                    xacc[0] = fmaf(e[2 * p], b0.x, fmaf(e[2 * p + 1], b1.x, xacc[0]));
                    xacc[1] = fmaf(e[2 * p], b0.y, fmaf(e[2 * p + 1], b1.y, xacc[1]));
                }
                split_pieces<NP>(a0.x, a1.x, a_p[0], p);
                split_pieces<NP>(a0.y, a1.y, a_p[1], p);
                split_pieces<NP>(b0.x, b1.x, b_p[0], p);
                split_pieces<NP>(b0.y, b1.y, b_p[1], p);
            }
        });
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c) mfma_pieces<NP>(a_p[a], b_p[c], acc[a][c]);
    };

    walk_column_list<Members, MODE == kKeySide>(csc_row, vals, gdb, beg, end,
                                                [&](int32_t jv, float, float, int first, Members& m) { fetch_members(jv, first, m); },
                                                [&](const Members& m, float gv, float ev, int first) { contract_members(m, gv, ev, first); });

    // the first tile's operand rows are requested here, with the splitting of the accumulators to cover the wait
    // (requested before the first contraction, they would hold 32 registers through it)
    float cn[4][8];
    float cfn = 1.0f;
    fetch_operand(row_cur, cn, cfn);

    // the extra row: lane f of either group holds columns 2f, 2f + 1
    float extra[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) extra[c] = xacc[c] + __shfl_xor(xacc[c], 32, kWave);

    // ---- the accumulators in pieces, in the registers' own order: [a][c][h] holds registers 8 h + 0..7
    uint32_t s_p[2][2][2][NP][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    split_pieces<NP>(acc[a][c][8 * h + 2 * p], acc[a][c][8 * h + 2 * p + 1], s_p[a][c][h], p);

    // ---- second contraction, 32 consumers at a time.  The consumer's own weight Phi_hat[i, l] is left to the
    // reduce kernel.
    const long long pbase = slice * static_cast<long long>(nnz);
    for (int32_t tile = beg; tile < end; tile += 32) {
        // this tile's operand, register 8 h + j of depth slot (g, j): element 2 (8 (2 h + j / 4) + 4 g + j % 4) + a
        float co[2][16];
        with_feature_map(fmap, [&](auto fm) {
            constexpr int FM = decltype(fm)::value;
#pragma unroll
            for (int hr = 0; hr < 4; ++hr)
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int a = 0; a < 2; ++a)
                        co[a][4 * hr + k] = MODE == kValueSide ? feature_ct<FM>(cn[hr][2 * k + a]) : cn[hr][2 * k + a];
        });
        const float coef = cfn;
        // next tile's operand rows, and the indices of the tile after it
        fetch_operand(row_next, cn, cfn);
        fetch_index(tile + 64, row_next);

        // register r of pc[c] is consumer tile + 8 (r / 4) + 4 g + r % 4, column 2 f + c
        floatx16 pc[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if constexpr (MODE == kQuerySide) {
                const float cr = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (8 * (r / 4) + 4 * g + (r % 4)), __float_as_int(coef)));
                pc[0][r] = cr * extra[0];
                pc[1][r] = cr * extra[1];
            } else if constexpr (MODE == kKeySide) {
                pc[0][r] = extra[0];
                pc[1][r] = extra[1];
            } else {
                pc[0][r] = 0.0f;
                pc[1][r] = 0.0f;
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t c_p[NP][4];
#pragma unroll
                for (int p = 0; p < 4; ++p) split_pieces<NP>(co[a][8 * h + 2 * p], co[a][8 * h + 2 * p + 1], c_p, p);
#pragma unroll
                for (int c = 0; c < 2; ++c) mfma_pieces<NP>(c_p, s_p[a][c][h], pc[c]);
            }

        store_consumer_tile(partial, pbase + tile, min(end - tile, 32), g, f, pc[0], pc[1]);
    }
    });
}

}  // namespace grf
