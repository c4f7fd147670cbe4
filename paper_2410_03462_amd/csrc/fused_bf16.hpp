// Bucket-fused evaluation (Eq. 7; Alg. 1 steps 3-5) for bf16 inputs at d = 64 on the bf16 matrix cores.
//
// The fp32 MFMA of gfx950 shares the vector ALU; v_mfma_f32_32x32x16_bf16 does not, and takes half the
// cycles for eight times the depth.  With bf16 inputs one operand of every product is a bf16 number as it
// stands (a row of V in the first contraction, a row of phi(Q) in the second: ReLU and the identity keep
// bf16 values bf16), and the other one (Phi_hat[j,l] phi(k_j), then S_l itself) is an fp32 number that is
// handed to the matrix cores as hi + lo, two bf16 numbers: hi the nearest bf16, lo the nearest bf16 of the
// rest, |x - hi - lo| <= 2^-16 |x|.  Products of bf16 numbers are exact in fp32 and all sums are fp32, so
// this is the fp32 kernel's arithmetic up to that 2^-16 on one operand.
//
// Index convention: MFMA row/column x of tile t stands for feature / value column 2x + t (a lane's two
// tiles are the two halves of one 32-bit word of a row).  Lane L = 32 g + f; in every operand the lanes of
// group g carry depth slots (g, 0..7) of the instruction, as two bf16 per register.
#pragma once

#include "split_common.hpp"

namespace grf {

// One wavefront per (slice, bucket l), one wavefront per workgroup.  Every global load is unconditional
// (members past the end of the column list re-read its last entry with weight 0).
//
// First contraction, 16 members of the list per step: lane (g, f) takes members 8 g + 0..7 of the step from
// the list block with ds_bpermute and loads word f of their rows of K and V (features / columns 2f, 2f + 1).
// The A tiles are Phi_hat[j,l] phi(k_j) as hi and lo, the B tiles the rows of V as stored, and a third B tile
// has ones in its column 0, so that z_l comes out as column 0 of a third accumulator tile, in the lanes and
// registers in which the second contraction needs it.
//
// Second contraction, 32 consumers per step: accumulator registers 8 h + 0..7 of tile (a, c), as hi and lo,
// are the B operand of depth slots (g, 0..7): S rows 2 (16 h + 8 (j / 4) + 4 g + j % 4) + a.  The A operand is
// consumer f's phi(q) at the same features: two 16-byte loads per h.  The partial denominator is the same
// product the other way round (the z tile as A, phi(Q) as B), which leaves it in register 0 of lanes 0..31.
template <bool WIDE, bool LISTED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void fused_bucket_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, long long n, int H, int n_f,
    const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row, const float* __restrict__ csc_val, int fmap,
    long long bh_first, long long n_waves, int32_t nnz, int spread_xcds, const int32_t* __restrict__ long_list,
    const int32_t* __restrict__ plan_counts, float* __restrict__ partial, float* __restrict__ pden)
{
    constexpr int D = 64;
    for_each_long_bucket<LISTED>(n, n_waves, spread_xcds, long_list, plan_counts, [&](uint32_t slice32, uint32_t l32) {
    const long long slice = slice32;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (static_cast<uint32_t>(bh) % static_cast<uint32_t>(H)) : 0u;
    const bf16_t* Qb = Q + bh * n * D;
    const bf16_t* Kb = K + bh * n * D;
    const bf16_t* Vb = V + bh * n * D;
    const float* vals = csc_val + plane * nnz;

    const int lane = lane_id();
    const int g = lane >> 5;
    const int f = lane & 31;

    const int32_t beg = __builtin_amdgcn_readfirstlane(col_ptr[l32]);
    const int32_t end = __builtin_amdgcn_readfirstlane(col_ptr[l32 + 1]);
    if (end - beg <= kGramMaxList) return;      // short lists (and empty ones) belong to gram_bucket_kernel

    const uint32_t floor16 = fmap == GRF_PHI_RELU ? 0u : 0x80008000u;

    // consumer f's phi(q) words for depth slots (g, .): features 2 rho, 2 rho + 1 for rho = 16 h + 8 run + 4 g + 0..3
    auto fetch_q = [&](int32_t row, uintx4 (&qw)[4]) {
#pragma unroll
        for (int hr = 0; hr < 4; ++hr)
            qw[hr] = *reinterpret_cast<const uintx4*>(row_elem_ptr<D, bf16_t, WIDE>(Qb, static_cast<uint32_t>(row), 2 * (8 * hr + 4 * g)));
    };
    auto fetch_index = [&](int32_t tile, int32_t& row) { row = csc_row[min(tile + f, end - 1)]; };

    // the first two consumer tiles' indices and the first tile's rows of Q go out before the first contraction
    int32_t qrow_cur, qrow_next;
    fetch_index(beg, qrow_cur);
    fetch_index(beg + 32, qrow_next);
    uintx4 qn[4];
    fetch_q(qrow_cur, qn);

    // ---- S_l = A^T V_l, z_l = A^T 1
    floatx16 acc[2][3];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
    const uint32_t one_pair = f == 0 ? 0x3f803f80u : 0u;      // bf16 1.0 twice
    const uint32_t ones_words[4] = {one_pair, one_pair, one_pair, one_pair};
    const bf16x8 b_ones = as_operand(ones_words);

    struct Members { uint32_t kw[8], vw[8]; float w[8]; };
    // members first + 8 g + 0..7 of the 64 entries held one per lane in (jv, gv)
    auto fetch_members = [&](int32_t jv, float gv, int first, Members& m) {
        int addr = 4 * ((first + 8 * g) & (kWave - 1));
        asm volatile("" : "+v"(addr));      // one register, the members' offsets as literals
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t row = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr + 4 * j, jv));
            m.w[j] = __int_as_float(__builtin_amdgcn_ds_bpermute(addr + 4 * j, __float_as_int(gv)));
            m.kw[j] = *reinterpret_cast<const uint32_t*>(row_elem_ptr<D, bf16_t, WIDE>(Kb, row, 2 * f));
            m.vw[j] = *reinterpret_cast<const uint32_t*>(row_elem_ptr<D, bf16_t, WIDE>(Vb, row, 2 * f));
        }
    };
    auto contract_members = [&](const Members& m) {
        uint32_t a_hi[2][4], a_lo[2][4], b_w[2][4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t kx = max_i16x2(m.kw[2 * p], floor16), ky = max_i16x2(m.kw[2 * p + 1], floor16);
            split_bf16(m.w[2 * p] * low_bf16(kx), m.w[2 * p + 1] * low_bf16(ky), a_hi[0][p], a_lo[0][p]);
            split_bf16(m.w[2 * p] * high_bf16(kx), m.w[2 * p + 1] * high_bf16(ky), a_hi[1][p], a_lo[1][p]);
            b_w[0][p] = low_halves(m.vw[2 * p], m.vw[2 * p + 1]);
            b_w[1][p] = high_halves(m.vw[2 * p], m.vw[2 * p + 1]);
        }
        const bf16x8 b_op[3] = {as_operand(b_w[0]), as_operand(b_w[1]), b_ones};
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const bf16x8 hi = as_operand(a_hi[a]), lo = as_operand(a_lo[a]);
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, b_op[c], acc[a][c], 0, 0, 0);
                acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, b_op[c], acc[a][c], 0, 0, 0);
            }
        }
    };

    walk_column_list<Members, false>(csc_row, vals, nullptr, beg, end,
                                     [&](int32_t jv, float gv, float, int first, Members& m) { fetch_members(jv, gv, first, m); },
                                     [&](const Members& m, float, float, int) { contract_members(m); });

    // ---- the accumulators as hi + lo, in the registers' own order: [a][c][h] holds registers 8 h + 0..7
    uint32_t s_hi[2][3][2][4], s_lo[2][3][2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 3; ++c)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    split_bf16(acc[a][c][8 * h + 2 * p], acc[a][c][8 * h + 2 * p + 1], s_hi[a][c][h][p], s_lo[a][c][h][p]);

    // ---- P_l = phi(Q_l) S_l and pden_l = phi(Q_l) z_l, 32 consumers at a time
    const long long pbase = slice * nnz;
    for (int32_t tile = beg; tile < end; tile += 32) {
        uint32_t aq[2][2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int run = 0; run < 2; ++run) {
                const uintx4 v = qn[2 * h + run];
                const uint32_t w0 = max_i16x2(v[0], floor16), w1 = max_i16x2(v[1], floor16);
                const uint32_t w2 = max_i16x2(v[2], floor16), w3 = max_i16x2(v[3], floor16);
                aq[0][h][2 * run] = low_halves(w0, w1);
                aq[0][h][2 * run + 1] = low_halves(w2, w3);
                aq[1][h][2 * run] = high_halves(w0, w1);
                aq[1][h][2 * run + 1] = high_halves(w2, w3);
            }
        // next tile's rows of Q, and the indices of the tile after it
        fetch_q(qrow_next, qn);
        fetch_index(tile + 64, qrow_next);

        floatx16 pc[2], pd;
#pragma unroll
        for (int r = 0; r < 16; ++r) { pc[0][r] = 0.0f; pc[1][r] = 0.0f; pd[r] = 0.0f; }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bf16x8 q_op = as_operand(aq[a][h]);
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    pc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q_op, as_operand(s_hi[a][c][h]), pc[c], 0, 0, 0);
                    pc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q_op, as_operand(s_lo[a][c][h]), pc[c], 0, 0, 0);
                }
                pd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(s_hi[a][2][h]), q_op, pd, 0, 0, 0);
                pd = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_operand(s_lo[a][2][h]), q_op, pd, 0, 0, 0);
            }
        if (g == 0 && tile + f < end) pden[pbase + tile + f] = pd[0];

        store_consumer_tile(partial, pbase + tile, min(end - tile, 32), g, f, pc[0], pc[1]);
    }
    });
}

}  // namespace grf
