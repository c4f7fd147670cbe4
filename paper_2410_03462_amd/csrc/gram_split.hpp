// Short column lists at d = 64: several buckets per wavefront, in Gram form, on the bf16 matrix cores.
//
// Per bucket l with contributor list C_l the fused forward pass (Eq. 7 with the shared features of Eq. 6) needs
//     P_l[i] = phi(q_i)^T S_l = sum_{j in C_l} w_j (phi(q_i) . phi(k_j)) v_j        for every i in C_l,
// and each backward pass a sum of the same shape.  Through S_l (d x d) that costs 4 r d^2 flops for a list of r
// entries; as (phi(Q_C) A^T) V_C, through the r x r matrix of dot products, it costs 4 r^2 d, which is less for
// r < d and far less for the lists of an image grid (about 7 entries), where a 16-member step and a 32-consumer
// tile of the S_l form are mostly padding.
//
// The entries of the column lists are consecutive in memory, bucket after bucket.  A work item is a run of at most 32
// consecutive entries that holds whole buckets only (planned by window_plan_kernel: the lists of at most kGramPackMax
// entries that start inside a run of 16 entries, together; a list of up to kGramMaxList entries alone), and a
// wavefront evaluates for it
//     E   = mask . (X_rows Y_rows^T)       32 x 32, depth d:   entry x entry dot products
//     out = E Z_rows                        32 x d,  depth 32
// where mask keeps the pairs of entries that belong to the same bucket (a block-diagonal matrix) and carries the
// members' weights.  Which rows X, Y, Z are depends on the pass:
//
//   pass          X (member m)   Y (consumer i)   E[m][i] before the mask        Z (member)    out_i
//   kForwardSide  phi(k_m)       phi(q_i)         w_m (x . y)                    v_m           P_l[i];  pden_i = sum_m E[m][i]
//   kQuerySide    v_m            g_i              w_m (x . y + gd_i)             phi(k_m)      U_i
//   kKeySide      g_m            v_i              w_m (x . y + gd_m)             phi(q_m)      R_i
//   kValueSide    phi(q_m)       phi(k_i)         w_m (x . y)                    g_m           X_i
//
// (g, gd: the rows of the backward seed, see backward.hip.)  Products are formed from bf16 pieces exactly as in the
// S_l kernels (three pieces and six products for fp32 inputs, two and three for bf16 inputs).
//
// Layout.  Lane L = 32 g + f.  First product: A operand = X rows, B operand = Y rows, both loaded the same way: lane
// (g, f) holds elements 16 s + 8 g + 0..7 of entry f's row for depth step s (32 contiguous bytes in fp32).  The
// result has member 8 (r / 4) + 4 g + r % 4 in register r and consumer f in the lane, which is, for registers
// 8 s + 0..7, the A operand of depth step s of the second product with depth slot (g, k) standing for member
// 16 s + 8 (k / 4) + 4 g + k % 4; the B operand takes the rows of Z at the same members, columns 2 f and 2 f + 1
// (MFMA column x of tile t stands for column 2 x + t, as in the S_l kernels).
#pragma once

#include "split_common.hpp"

namespace grf {

// One wavefront per workgroup, as many workgroups as are resident at once; a wavefront works through the items
// t, t + stride, ... of all (slice, item) pairs.  Two items are in flight besides the current one: the next one's
// list entries are requested while the current item's rows are on their way, and the range of the one after with
// them, so that an item starts with one memory round trip (its rows) instead of three.
template <typename T, int MODE, bool WIDE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3))) void gram_bucket_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const float* __restrict__ G, const float* __restrict__ gd,
    long long n, int H, int n_f, const int2* __restrict__ items, const int32_t* __restrict__ plan_counts,
    const int32_t* __restrict__ csc_row, const int32_t* __restrict__ csc_span, const float* __restrict__ csc_val, int fmap,
    long long bh_first, uint32_t n_slices, int32_t nnz, int spread_xcds, float* __restrict__ partial, float* __restrict__ pden)
{
    constexpr int D = 64;
    constexpr int NP = sizeof(T) == 2 ? 2 : 3;
    typedef typename std::conditional<MODE == kKeySide, float, T>::type TX;
    typedef typename std::conditional<MODE == kQuerySide, float, T>::type TY;
    typedef typename std::conditional<MODE == kValueSide, float, T>::type TZ;
    constexpr bool PHI_XY = MODE == kForwardSide || MODE == kValueSide;      // else the feature map sits on Z

    const uint32_t count = static_cast<uint32_t>(plan_counts[kPlanItems]);     // items per slice
    if (count == 0) return;
    const uint32_t all = n_slices * count;      // < 2^31, checked by the host against the plan's capacity
    // which (slice, item) pairs this wavefront takes: see fused_bucket_kernel for the two ways of sharing them out
    uint32_t t, stride = gridDim.x, total = all;
    if (spread_xcds) {
        const uint32_t parts = min(8u, gridDim.x);
        const uint32_t xcd = blockIdx.x % parts;
        const uint32_t share = all / parts, extra = all % parts;
        const uint32_t first = xcd * share + min(xcd, extra);
        total = first + share + (xcd < extra ? 1u : 0u);
        stride = (gridDim.x - xcd + parts - 1) / parts;
        t = first + blockIdx.x / parts;
    } else {
        t = static_cast<uint32_t>(xcd_contiguous_block(blockIdx.x, gridDim.x));
    }
    if (t >= total) return;
    struct Position { uint32_t t, slice, i; };
    const uint32_t step_slices = stride / count, step_items = stride % count;      // one division per wavefront
    auto after = [&](Position p) {
        p.t += stride;
        p.slice += step_slices;
        p.i += step_items;
        if (p.i >= count) { p.i -= count; ++p.slice; }
        return p;
    };

    const int lane = lane_id();
    const int g = lane >> 5;
    const int f = lane & 31;
    int slot0 = 16 * g;
    asm volatile("" : "+v"(slot0));      // one register, the members' offsets as literals
    // member of depth slot (g, k) of step s of the second product, as a ds_bpermute address
    auto member_addr = [&](int s, int k) { return slot0 + 4 * (16 * s + 8 * (k / 4) + (k % 4)); };

    // an item's range, through the vector memory path (the same address in every lane) so that it is counted with
    // the other loads in issue order; past the wavefront's last item the last valid one is re-read and not used
    auto range_of = [&](const Position& p) {
        uint32_t idx = min(p.i, count - 1);
        asm volatile("" : "+v"(idx));
        return items[idx];
    };
    // entry f of an item (both half-waves hold it); lanes past its end re-read its last entry
    struct Entries { int32_t row, span; float w, gd; };
    auto entries_of = [&](const Position& p, int2 range) {
        const int32_t cnt = max(min(range.y - range.x, kGramTile), 1);
        const int32_t e = range.x + min(f, cnt - 1);
        const uint32_t bh = static_cast<uint32_t>(bh_first) + min(p.slice, n_slices - 1);
        const long long plane = n_f > 1 ? (bh % static_cast<uint32_t>(H)) : 0u;
        Entries en;
        en.row = csc_row[e];
        en.span = csc_span[e];
        en.w = csc_val[plane * nnz + e];
        en.gd = 0.0f;
        if constexpr (MODE == kQuerySide || MODE == kKeySide)
            en.gd = gd[static_cast<long long>(min(p.slice, n_slices - 1)) * n + static_cast<uint32_t>(en.row)];
        return en;
    };

    Position cur;
    cur.t = t;
    cur.slice = t / count;
    cur.i = t - cur.slice * count;
    Position nxt = after(cur);
    int2 range_cur = range_of(cur);
    int2 range_nxt = range_of(nxt);
    Entries en_cur = entries_of(cur, range_cur);

    with_feature_map(fmap, [&](auto fm) {
        constexpr int FM = decltype(fm)::value;
        for (;;) {
            const int32_t e0 = __builtin_amdgcn_readfirstlane(range_cur.x);
            const int32_t cnt = max(min(__builtin_amdgcn_readfirstlane(range_cur.y) - e0, kGramTile), 1);
            const long long slice = cur.slice;
            const long long row0 = (bh_first + slice) * n * D;
            const float* Gb = G + slice * n * D;
            const TX* Xb; const TY* Yb; const TZ* Zb;
            if constexpr (MODE == kForwardSide) { Xb = K + row0; Yb = Q + row0; Zb = V + row0; }
            if constexpr (MODE == kQuerySide) { Xb = V + row0; Yb = Gb; Zb = K + row0; }
            if constexpr (MODE == kKeySide) { Xb = Gb; Yb = V + row0; Zb = Q + row0; }
            if constexpr (MODE == kValueSide) { Xb = Q + row0; Yb = K + row0; Zb = Gb; }

            const uint32_t row_f = static_cast<uint32_t>(en_cur.row);
            const float w_f = f < cnt ? en_cur.w : 0.0f;      // past the end: weight 0 and outside every bucket
            const int32_t start_f = f - (en_cur.span & 0xff);     // window positions [start_f, start_f + len_f) are f's bucket
            const int32_t len_f = f < cnt ? en_cur.span >> 8 : 0;
            const float gd_f = en_cur.gd;

            // ---- this item's rows, then the next item's entries and the range of the one after
            float x[4][8], y[4][8];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                load_eight<TX, WIDE>(Xb, row_f, 16 * s + 8 * g, x[s]);
                load_eight<TY, WIDE>(Yb, row_f, 16 * s + 8 * g, y[s]);
            }
            const Position nn = after(nxt);
            const Entries en_nxt = entries_of(nxt, range_nxt);
            const int2 range_nn = range_of(nn);
            typename RawPair<TZ>::type z[2][8];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t row_m = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(member_addr(s, k), static_cast<int>(row_f)));
                    z[s][k] = load_pair<TZ, WIDE>(Zb, row_m, f);
                }
            __builtin_amdgcn_sched_barrier(0);

            // ---- first product: entry x entry dot products
            floatx16 dots;
#pragma unroll
            for (int r = 0; r < 16; ++r) dots[r] = 0.0f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint32_t x_p[NP][4], y_p[NP][4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    if constexpr (PHI_XY) {
                        split_pieces<NP>(feature_ct<FM>(x[s][2 * p]), feature_ct<FM>(x[s][2 * p + 1]), x_p, p);
                        split_pieces<NP>(feature_ct<FM>(y[s][2 * p]), feature_ct<FM>(y[s][2 * p + 1]), y_p, p);
                    } else {
                        split_pieces<NP>(x[s][2 * p], x[s][2 * p + 1], x_p, p);
                        split_pieces<NP>(y[s][2 * p], y[s][2 * p + 1], y_p, p);
                    }
                }
                mfma_pieces<NP>(x_p, y_p, dots);
            }

            // ---- mask and weights: register r is member 8 (r / 4) + 4 g + r % 4, the lane is consumer f
            float em[16];
            const float wgd_f = w_f * gd_f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int addr = member_addr(r / 8, r % 8);
                const int m = 8 * (r / 4) + 4 * g + (r % 4);
                const float w_m = __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(w_f)));
                float v;
                if constexpr (MODE == kQuerySide) v = (dots[r] + gd_f) * w_m;
                else if constexpr (MODE == kKeySide) v = fmaf(dots[r], w_m, __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(wgd_f))));
                else v = dots[r] * w_m;
                em[r] = static_cast<uint32_t>(m - start_f) < static_cast<uint32_t>(len_f) ? v : 0.0f;
            }
            const long long pbase = slice * static_cast<long long>(nnz) + e0;
            if constexpr (MODE == kForwardSide) {
                float dsum = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) dsum += em[r];
                dsum += __shfl_xor(dsum, 32, kWave);
                if (g == 0 && f < cnt) pden[pbase + f] = dsum;
            }

            // ---- second product
            floatx16 p0, p1;
#pragma unroll
            for (int r = 0; r < 16; ++r) { p0[r] = 0.0f; p1[r] = 0.0f; }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                uint32_t e_p[NP][4], z0_p[NP][4], z1_p[NP][4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    split_pieces<NP>(em[8 * s + 2 * p], em[8 * s + 2 * p + 1], e_p, p);
                    float2 za = widen(z[s][2 * p]), zb = widen(z[s][2 * p + 1]);
                    if constexpr (!PHI_XY) {
                        za = make_float2(feature_ct<FM>(za.x), feature_ct<FM>(za.y));
                        zb = make_float2(feature_ct<FM>(zb.x), feature_ct<FM>(zb.y));
                    }
                    split_pieces<NP>(za.x, zb.x, z0_p, p);
                    split_pieces<NP>(za.y, zb.y, z1_p, p);
                }
                mfma_pieces<NP>(e_p, z0_p, p0);
                mfma_pieces<NP>(e_p, z1_p, p1);
            }

            // register r of p0 / p1 is consumer 8 (r / 4) + 4 g + r % 4, columns 2 f and 2 f + 1
            store_consumer_tile(partial, pbase, cnt, g, f, p0, p1);

            if (nxt.t >= total) break;
            cur = nxt; nxt = nn;
            range_cur = range_nxt; range_nxt = range_nn;
            en_cur = en_nxt;
        }
    });
}

}  // namespace grf
