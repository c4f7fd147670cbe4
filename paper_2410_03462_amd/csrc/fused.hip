// Bucket-fused evaluation of GRF-masked linear attention (Eq. 7; Alg. 1 steps 3-5): the same
// num, den, out as the bucket + gather pair, but S_l never leaves the registers.
//
// Queries and keys use the same graph features (Eq. 6), so the rows that consume bucket l are
// exactly the rows that contribute to it: the column list C_l of Phi_hat.  Per bucket,
//     S_l = A^T V_l,            A = diag(Phi_hat[C_l, l]) phi(K[C_l])      (r_l x d)
//     P_l = phi(Q[C_l]) S_l                                                 (r_l x d)
//     pden_l = phi(Q[C_l]) z_l,  z_l = A^T 1
// and then num_i = sum_l Phi_hat[i,l] P_l[i], den_i = sum_l Phi_hat[i,l] pden_l[i] over the entries of
// row i.  Both contractions run on v_mfma_f32_32x32x2_f32; P_l and pden_l are streamed out in
// column-list order (one d-float row per entry of Phi_hat) and a second kernel forms each row's
// weighted sums in ascending-l order, so the result is deterministic and no float atomics are used.
// (The consumer's weight is applied there because the second kernel is bound by memory, whereas every
// vector instruction of this one is paid in matrix time.)
//
// Index convention (T2 = d/32): MFMA row/column x of tile t stands for feature / value column
// T2*x + t, so that a lane's T2 operands are adjacent in memory (one 8-byte load at d = 64).
#include <mutex>

#include "attention_common.hpp"
#include "fused_bf16.hpp"
#include "fused_split.hpp"
#include "gram_split.hpp"

namespace grf {

// One wavefront per workgroup, each working through the (slice, bucket) pairs w, w + G, w + 2G, ... of a grid
// of G resident wavefronts: column lists differ in length, and the next bucket's bounds and first list block
// are fetched while the current bucket is still in its matrix work, so that a bucket does not start with a
// chain of three dependent memory round trips (bounds, list, rows).
//
// Every global load below is unconditional: lanes past the end of the column list re-read its last
// entry with weight 0, so there are no branches around loads and the loads of the next stage
// (next group of K/V rows, next tile's Q rows, the indices after that) are issued before the
// matrix work of the current stage and waited for only afterwards.
template <int D, typename T, bool WIDE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void fused_bucket_kernel(const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
                                                           long long n, int H, int n_f,
                                                           const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row,
                                                           const float* __restrict__ csc_val,
                                                           int fmap, long long bh_first, long long n_waves, int32_t nnz,
                                                           int spread_xcds, float* __restrict__ partial, float* __restrict__ pden)
{
    constexpr int T2 = D / 32;
    constexpr int QN = 4 * T2;     // features a lane holds per group of four accumulator registers
    // B*H*n < 2^31 (checked by the host), so the bucket counter fits 32 bits.  A wavefront divides once, for its first
    // bucket, and then steps (slice, l) along by the grid size: a 64-bit division per bucket costs about a
    // microsecond of dependent scalar instructions, which is a tenth of a short bucket's whole work.
    struct Position { uint32_t wave, slice, l; };
    const uint32_t n32 = static_cast<uint32_t>(n);
    // Workgroups go to the eight XCDs round-robin by id.  Two ways of sharing out the buckets, chosen by the host:
    //   spread_xcds   each XCD takes one contiguous eighth of all buckets and its resident wavefronts stride through
    //                 it, so the XCDs work in different slices: their row reads do not all land on the same lines of
    //                 the memory side.  Right when eight slices' Q, K, V fit the Infinity Cache with room to spare.
    //   otherwise     the grid strides through all buckets together, each XCD holding a contiguous run of the buckets
    //                 in flight: one slice's Q, K, V are hot at a time.
    const uint32_t all = static_cast<uint32_t>(n_waves);
    uint32_t total = all, stride = gridDim.x;
    Position cur;
    if (spread_xcds) {
        const uint32_t parts = min(8u, gridDim.x);      // XCDs that receive workgroups of this grid
        const uint32_t xcd = blockIdx.x % parts;
        const uint32_t share = all / parts, extra = all % parts;
        const uint32_t first_bucket = xcd * share + min(xcd, extra);
        total = first_bucket + share + (xcd < extra ? 1u : 0u);      // end of this XCD's range
        stride = (gridDim.x - xcd + parts - 1) / parts;               // workgroups of this grid on this XCD
        cur.wave = first_bucket + blockIdx.x / parts;
    } else {
        cur.wave = static_cast<uint32_t>(xcd_contiguous_block(blockIdx.x, gridDim.x));
    }
    if (cur.wave >= total) return;
    cur.slice = cur.wave / n32;
    cur.l = cur.wave - cur.slice * n32;
    auto after = [&](Position p) {
        p.wave += stride;
        p.l += stride;
        while (p.l >= n32) { p.l -= n32; ++p.slice; }
        return p;
    };

    const int lane = lane_id();
    const int half = lane >> 5;
    const int li = lane & 31;

    // bounds of a bucket's column list; an empty list past the wavefront's last bucket.  The index is the same in
    // every lane, so these are scalar loads.
    auto bounds_of = [&](const Position& p, int32_t& beg, int32_t& end) {
        beg = 0; end = 0;
        if (p.wave < total) { beg = col_ptr[p.l]; end = col_ptr[p.l + 1]; }
    };
    auto values_of = [&](uint32_t sl) {
        const uint32_t bh = static_cast<uint32_t>(bh_first) + sl;
        return csc_val + (n_f > 1 ? (bh % static_cast<uint32_t>(H)) : 0u) * static_cast<long long>(nnz);
    };

    // Three buckets are in flight per wavefront: the one being worked on, the next one, whose first list block is
    // requested before the current bucket's own loads, and the one after, whose bounds are requested with it.  What
    // was requested is taken into registers right after the first contraction, where the in-order load counter has
    // long passed it: left until the next bucket starts, it would be waited for behind a run of stores whose length
    // the compiler cannot know, that is, with a wait for every outstanding store.
    Position nxt = after(cur);
    int32_t beg, end, beg1, end1;
    bounds_of(cur, beg, end);
    bounds_of(nxt, beg1, end1);
    ListBlock first = load_list_block<false>(csc_row, values_of(cur.slice), nullptr, beg, end);

    for (;;) {
        const uint32_t slice = cur.slice;
        const long long bh = bh_first + slice;
        const T* Qb = Q + bh * n * D;
        const T* Kb = K + bh * n * D;
        const T* Vb = V + bh * n * D;
        const float* vals = values_of(slice);

        const Position nn = after(nxt);
        int32_t beg2, end2;
        bounds_of(nn, beg2, end2);
        ListBlock first_next = load_list_block<false>(csc_row, values_of(nxt.slice), nullptr, beg1, end1);

        if (beg >= end) {      // nobody visits this node: no partial rows belong to it
            if (nxt.wave >= total) break;
            asm volatile("" : "+v"(first_next.j_a), "+v"(first_next.j_b), "+v"(first_next.g_a), "+v"(first_next.g_b));
            cur = nxt; nxt = nn;
            beg = beg1; end = end1; beg1 = beg2; end1 = end2;
            first = first_next;
            continue;
        }

        // consumers of tile `tile`: row index of entry tile + li (clamped to the last entry)
        auto fetch_index = [&](int32_t tile, int32_t& row) { row = csc_row[min(tile + li, end - 1)]; };
        auto fetch_q = [&](int32_t row, float (&qq)[4][QN]) {
            const T* p = row_elem_ptr<D, T, WIDE>(Qb, static_cast<uint32_t>(row), T2 * 4 * half);
#pragma unroll
            for (int b = 0; b < 4; ++b) load_run<T, QN>(p + T2 * 8 * b, qq[b]);
        };

        // the first two consumer tiles are entries beg .. beg + 63 of the list, which the first block holds (one
        // per lane); the first tile's rows of Q go out before the first contraction starts
        int32_t qrow_cur = __shfl(first.j_a, li, kWave), qrow_next = __shfl(first.j_a, 32 + li, kWave);
        float qn[4][QN];
        fetch_q(qrow_cur, qn);

        // ---- S_l = A^T V_l
        floatx16 acc[T2][T2];
        float zacc[T2];
        with_feature_map(fmap, [&](auto fm) {
            bucket_first_contraction<D, T, T, true, true, kExtraSumA, decltype(fm)::value, WIDE>(Kb, Vb, csc_row, vals, nullptr, beg, end, first, acc, zacc);
        });

        // the next bucket's first list block and the bounds after it have arrived: into registers now (see above)
        asm volatile("" : "+v"(first_next.j_a), "+v"(first_next.j_b), "+v"(first_next.g_a), "+v"(first_next.g_b));
        beg2 = __builtin_amdgcn_readfirstlane(beg2);
        end2 = __builtin_amdgcn_readfirstlane(end2);

        float zfull[T2];
#pragma unroll
        for (int t = 0; t < T2; ++t) zfull[t] = zacc[t] + __shfl_xor(zacc[t], 32, kWave);

        // ---- P_l = phi(Q_l) S_l, 32 consumers at a time.  Accumulator register r of tile (t, c) holds
        // S[T2*(8*(r/4) + 4*half + r%4) + t][T2*li + c]: fed back unchanged as the B operand, it pairs the
        // feature held by the lower half-wave (k = 0) with the one held by the upper (k = 1); the A operand
        // takes the same two features of consumer li's phi(q).
        const long long pbase = static_cast<long long>(slice) * nnz;
        for (int32_t tile = beg; tile < end; tile += 32) {
            float qv[4][QN];
            with_feature_map(fmap, [&](auto fm) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int e2 = 0; e2 < QN; ++e2) qv[b][e2] = feature_ct<decltype(fm)::value>(qn[b][e2]);
            });
            // next tile's rows of Q, and the indices of the tile after it
            fetch_q(qrow_next, qn);
            fetch_index(tile + 64, qrow_next);

            __builtin_amdgcn_sched_barrier(0);

            // 4*T2 MFMAs per accumulator register r of S, and the two terms of the partial denominator that use
            // the same features: phi(q) against z_l, which sits in the lanes in the order of the first
            // contraction's rows.
            floatx16 pc[T2];
#pragma unroll
            for (int c = 0; c < T2; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) pc[c][r] = 0.0f;
            float dl = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
#pragma unroll
                for (int t = 0; t < T2; ++t) {
#pragma unroll
                    for (int c = 0; c < T2; ++c)
                        pc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(qv[r / 4][T2 * (r % 4) + t], acc[t][c][r], pc[c], 0, 0, 0);
                    dl = fmaf(qv[r / 4][T2 * (r % 4) + t], __shfl(zfull[t], 8 * (r / 4) + 4 * half + (r % 4), kWave), dl);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            dl += __shfl_xor(dl, 32, kWave);
            if (half == 0 && tile + li < end) pden[pbase + tile + li] = dl;

            // register r of pc[c] is consumer tile + 8*(r/4) + 4*half + r%4, column T2*li + c: stored through a
            // window over the tile's rows, which drops the rows past the end of the list
            const __amdgpu_buffer_rsrc_t window = row_window(partial, pbase + tile, min(end - tile, 32), D);
            // opaque here so that the rows' constant offsets are formed next to the stores, where they fold into the
            // instructions' offset fields (hoisted out of the loop they would occupy 16*T2 registers)
            int lane_off = (4 * half * D + T2 * li) * 4;
            asm volatile("" : "+v"(lane_off));
            // the whole offset goes through the vector offset and the instruction's offset field, the two terms that
            // the range check covers.  One column tile after the other, kept apart: merged into 8-byte stores, the
            // two tiles' registers (never adjacent) would have to be copied next to each other first
#pragma unroll
            for (int c = 0; c < T2; ++c) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(pc[c][r]), window, lane_off + (8 * (r / 4) + (r % 4)) * D * 4 + 4 * c, 0, 0);
                asm volatile("" ::: "memory");
            }
        }
        if (nxt.wave >= total) break;
        cur = nxt; nxt = nn;
        beg = beg1; end = end1; beg1 = beg2; end1 = end2;
        first = first_next;
    }
}

// One wavefront per (slice, row i): sums the row's partial numerators and denominators, each times its
// entry Phi_hat[i, l], in ascending-l order and divides.
template <int D>
__global__ __launch_bounds__(256) void fused_reduce_kernel(long long n, int H, int n_f, long long val_stride,
                                                           const int32_t* __restrict__ row_ptr, const float* __restrict__ phi_val,
                                                           const int32_t* __restrict__ csr_to_csc, int32_t nnz,
                                                           const float* __restrict__ partial, const float* __restrict__ pden,
                                                           long long bh_first, long long n_waves,
                                                           float* __restrict__ out, float* __restrict__ num_opt, float* __restrict__ den_opt)
{
    constexpr int EPW = kWave / D;     // entries per wavefront step (1 at d = 64, 2 at d = 32)
    const long long wave = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long i = wave - slice * n;
    const long long bh = bh_first + slice;
    const int lane = lane_id();
    const int sub = lane / D;
    const int c = lane % D;
    const float* slice_partial = partial + slice * static_cast<long long>(nnz) * D;
    const float* slice_pden = pden + slice * static_cast<long long>(nnz);
    const float* vals = phi_val + (n_f > 1 ? (bh % H) : 0) * val_stride;

    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    float acc = 0.0f, dacc = 0.0f;
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        const int32_t pos_reg = e < end ? csr_to_csc[e] : -1;
        const float w_reg = e < end ? vals[e] : 0.0f;
        const int cnt = min(kWave, end - chunk);
        // eight entries' loads are issued together; the shuffles are executed by every lane (a
        // disabled source lane would read as 0)
        for (int t0 = 0; t0 < cnt; t0 += 8 * EPW) {
            float v[8], dv[8], w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = t0 + u * EPW + sub;
                if constexpr (EPW == 1) {
                    // the entry is the same in every lane: scalar broadcasts, a row address in scalar registers and a
                    // scalar load of the partial denominator; the loads are unconditional
                    const int32_t pos = __builtin_amdgcn_readlane(pos_reg, t & (kWave - 1));
                    w[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_reg), t & (kWave - 1)));
                    const bool ok = t < cnt && pos >= 0;
                    const float x = slice_partial[static_cast<long long>(max(pos, 0)) * D + c];
                    const float dx = slice_pden[max(pos, 0)];
                    v[u] = ok ? x : 0.0f;
                    dv[u] = ok ? dx : 0.0f;
                } else {
                    const int32_t pos = __shfl(pos_reg, t & (kWave - 1), kWave);
                    w[u] = __shfl(w_reg, t & (kWave - 1), kWave);
                    const bool ok = t < cnt && pos >= 0;
                    v[u] = ok ? slice_partial[static_cast<long long>(pos) * D + c] : 0.0f;
                    dv[u] = ok ? slice_pden[pos] : 0.0f;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc = fmaf(w[u], v[u], acc); dacc = fmaf(w[u], dv[u], dacc); }
        }
    }
    if constexpr (EPW == 2) {
        acc += __shfl_xor(acc, 32, kWave);
        dacc += __shfl_xor(dacc, 32, kWave);
    }
    if (sub == 0) {
        const long long o = (bh * n + i) * D + c;
        out[o] = acc / dacc;
        if (num_opt != nullptr) num_opt[o] = acc;
        if (c == 0 && den_opt != nullptr) den_opt[bh * n + i] = dacc;
    }
}

namespace {

template <int D, typename T>
grf_status launch_fused(const void* Q, const void* K, const void* V, int64_t n, int64_t H, int32_t n_f, const grf_phi* phi,
                        int64_t nnz, const Transposed& t, int fmap, int64_t bh_first, int64_t n_slices,
                        float* partial, float* pden, float* out, float* num_opt, float* den_opt, hipStream_t stream)
{
    const long long waves = static_cast<long long>(n_slices) * n;
    if (waves == 0) return GRF_OK;
    if (D == 64 && static_cast<long long>(n_slices) * t.item_capacity >= 2147483647ll)
        return fail(GRF_EUNSUPPORTED, "slices * nnz / 8 = %lld * %lld must be < 2^31", (long long)n_slices, t.item_capacity);
    // eight slices' Q, K, V within a quarter of the 256 MB Infinity Cache: see the kernel
    const int spread = 8ll * 3 * n * D * static_cast<long long>(sizeof(T)) <= (64ll << 20) ? 1 : 0;
    auto launch = [&](auto wide) {
        constexpr bool W = decltype(wide)::value;
        if constexpr (D == 64) {
            // d = 64 runs on the bf16 matrix cores: bf16 inputs under a feature map that keeps bf16 values bf16 with
            // two-piece fp32 operands, everything else with three-piece operands and six products
            // lists of at most kGramMaxList entries, several buckets per wavefront; the kernels below skip them
            hipLaunchKernelGGL((gram_bucket_kernel<T, kForwardSide, W>),
                               dim3(resident_wave_grid(reinterpret_cast<const void*>(&gram_bucket_kernel<T, kForwardSide, W>), static_cast<long long>(n_slices) * t.item_capacity)),
                               dim3(kWave), 0, stream,
                               static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                               static_cast<const float*>(nullptr), static_cast<const float*>(nullptr),
                               static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f),
                               static_cast<const int2*>(t.items), static_cast<const int32_t*>(t.plan_counts),
                               static_cast<const int32_t*>(t.s_row), static_cast<const int32_t*>(t.span),
                               static_cast<const float*>(t.s_val), fmap, static_cast<long long>(bh_first),
                               static_cast<uint32_t>(n_slices), static_cast<int32_t>(nnz), spread, partial, pden);
            // the longer lists: one workgroup per bucket when most lists are long, else a resident grid over the listed ones
            auto go = [&](auto kernel, bool listed) {
                const unsigned grid = listed ? resident_wave_grid(reinterpret_cast<const void*>(kernel), waves) : static_cast<unsigned>(waves);
                hipLaunchKernelGGL(kernel, dim3(grid), dim3(kWave), 0, stream,
                                   static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                                   static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f),
                                   static_cast<const int32_t*>(t.col_ptr), static_cast<const int32_t*>(t.s_row),
                                   static_cast<const float*>(t.s_val), fmap, static_cast<long long>(bh_first), waves,
                                   static_cast<int32_t>(nnz), spread, static_cast<const int32_t*>(t.long_list),
                                   static_cast<const int32_t*>(t.plan_counts), partial, pden);
            };
            const bool listed = few_long_lists(n, nnz);
            if constexpr (std::is_same<T, bf16_t>::value) {
                if (fmap != GRF_PHI_ELU1) {
                    if (listed) go(fused_bucket_bf16_kernel<W, true>, true); else go(fused_bucket_bf16_kernel<W, false>, false);
                    return;
                }
            }
            if (listed) go(fused_bucket_split_kernel<T, W, true>, true); else go(fused_bucket_split_kernel<T, W, false>, false);
        } else {
            hipLaunchKernelGGL((fused_bucket_kernel<D, T, W>), dim3(resident_wave_grid(reinterpret_cast<const void*>(&fused_bucket_kernel<D, T, W>), waves)), dim3(kWave), 0, stream,
                               static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                               static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f),
                               static_cast<const int32_t*>(t.col_ptr), static_cast<const int32_t*>(t.s_row),
                               static_cast<const float*>(t.s_val), fmap, static_cast<long long>(bh_first), waves,
                               static_cast<int32_t>(nnz), spread, partial, pden);
        }
    };
    if (wide_offsets(n, D)) launch(std::true_type{}); else launch(std::false_type{});
    GRF_LAUNCH_CHECK("fused_bucket_kernel");
    hipLaunchKernelGGL((fused_reduce_kernel<D>), dim3(blocks_for(waves, 4)), dim3(256), 0, stream,
                       static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f), static_cast<long long>(phi->capacity),
                       static_cast<const int32_t*>(phi->row_ptr), static_cast<const float*>(phi->val),
                       static_cast<const int32_t*>(t.csr_to_csc), static_cast<int32_t>(nnz),
                       static_cast<const float*>(partial), static_cast<const float*>(pden),
                       static_cast<long long>(bh_first), waves, out, num_opt, den_opt);
    GRF_LAUNCH_CHECK("fused_reduce_kernel");
    return GRF_OK;
}

size_t partial_bytes(int64_t slices, int64_t nnz, int32_t d) { return align_up(sizeof(float) * static_cast<size_t>(slices) * static_cast<size_t>(nnz > 0 ? nnz : 1) * d); }
size_t pden_bytes(int64_t slices, int64_t nnz) { return align_up(sizeof(float) * static_cast<size_t>(slices) * static_cast<size_t>(nnz > 0 ? nnz : 1)); }

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" size_t grf_fused_attention_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk)
{
    if (B < 0 || H < 0 || n < 0 || nnz < 0 || n_f < 1 || (d != 32 && d != 64)) return 0;
    int64_t slices = B * H;
    if (bh_chunk > 0 && bh_chunk < slices) slices = bh_chunk;
    return carve_transposed(nullptr, n, nnz, n_f).bytes + partial_bytes(slices, nnz, d) + pden_bytes(slices, nnz);
}

namespace {

// The bucket-fused entry points behind their argument checks: bucket kernels + row reduction per chunk of `step`
// slices over the column lists `t`; `rest` holds the partial rows and partial denominators of one chunk.
grf_status fused_chunks(const void* Q, const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                        const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map, int64_t step, const Transposed& t,
                        unsigned char* rest, hipStream_t stream, float* out, float* num_opt, float* den_opt)
{
    const int64_t slices = B * H;
    float* partial = reinterpret_cast<float*>(rest);
    float* pden = reinterpret_cast<float*>(rest + partial_bytes(step, nnz, d));
    const int fmap = feature_map;
    for (int64_t first = 0; first < slices; first += step) {
        const int64_t count = (slices - first < step) ? (slices - first) : step;
        grf_status st = GRF_OK;
        GRF_DISPATCH(d, dtype, (st = launch_fused<D_, T_>(Q, K, V, n, H, n_f, phi, nnz, t, fmap, first, count, partial, pden,
                                                          out, num_opt, den_opt, stream)));
        if (st != GRF_OK) return st;
    }
    return GRF_OK;
}

// Column lists built at the head of `ws` (grf_fused_attention_workspace_bytes(..., step) bytes), then the chunks.
grf_status fused_impl(const void* Q, const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                      const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map, int64_t step,
                      unsigned char* ws, hipStream_t stream, float* out, float* num_opt, float* den_opt)
{
    const Transposed t = carve_transposed(ws, n, nnz, n_f);
    if (grf_status st = transpose(phi, nnz, n_f, t, stream)) return st;
    return fused_chunks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, step, t, ws + t.bytes, stream, out, num_opt, den_opt);
}

}  // namespace

extern "C" grf_status grf_masked_linear_attention_fused_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
                                                                 int64_t B, int64_t H, int64_t n, int32_t d,
                                                                 const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                                 int32_t bh_chunk, const void* prepared, size_t prepared_bytes,
                                                                 void* workspace, size_t workspace_bytes, void* hip_stream,
                                                                 float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr)) return fail(GRF_EINVAL, "Q / out is NULL");
    Transposed t;
    if (grf_status st = prepared_lists(prepared, prepared_bytes, n, nnz, n_f, &t)) return st;
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    if (grf_status st = check_workspace(workspace, workspace_bytes, partial_bytes(step, nnz, d) + pden_bytes(step, nnz))) return st;
    if (B * H * n == 0) return GRF_OK;
    return fused_chunks(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, step, t, static_cast<unsigned char*>(workspace),
                        static_cast<hipStream_t>(hip_stream), out, num_opt, den_opt);
}

extern "C" grf_status grf_masked_linear_attention_fused(const void* Q, const void* K, const void* V, int32_t dtype,
                                                        int64_t B, int64_t H, int64_t n, int32_t d,
                                                        const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                        int32_t bh_chunk,
                                                        void* workspace, size_t workspace_bytes, void* hip_stream,
                                                        float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr)) return fail(GRF_EINVAL, "Q / out is NULL");
    if (grf_status st = check_workspace(workspace, workspace_bytes, grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))) return st;
    if (B * H * n == 0) return GRF_OK;
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    return fused_impl(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, step, static_cast<unsigned char*>(workspace),
                      static_cast<hipStream_t>(hip_stream), out, num_opt, den_opt);
}

// ------------------------------------------------------------------------------------ the call that allocates nothing
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid hipMalloc) and hold no
// workspace either: the column lists and the per-entry partial rows live in a device array that is part of the
// loaded library.  Every GPU the library runs on holds its own copy of the array until the process ends.
constexpr size_t kStaticScratchBytes = 64ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once asked for

// Device address of the scratch array on the current device.  `scratch` itself is only a host-side handle of the
// symbol; host code must never use it as an address.
grf_status static_scratch(unsigned char** ptr)
{
    int device = -1;
    GRF_HIP_TRY(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return fail(GRF_EUNSUPPORTED, "device ordinal %d is outside [0, %d)", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        GRF_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) % kAlign) != 0)
            return fail(GRF_EHIP, "hipGetSymbolAddress gave %p for the static scratch array", p);
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *ptr = g_scratch_ptr[device];
    return GRF_OK;
}

}  // namespace

extern "C" grf_status grf_masked_linear_attention_fused_static(const void* Q, const void* K, const void* V, int32_t dtype,
                                                               int64_t B, int64_t H, int64_t n, int32_t d,
                                                               const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                               void* hip_stream, float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr)) return fail(GRF_EINVAL, "Q / out is NULL");
    if (B * H * n == 0) return GRF_OK;
    // as many slices per chunk as the array holds (results do not depend on the chunking)
    const int64_t slices = B * H;
    const size_t one = grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, 1);
    if (one == 0 || one > kStaticScratchBytes)
        return fail(GRF_EUNSUPPORTED, "one slice needs %zu bytes of scratch (grf_fused_attention_workspace_bytes with bh_chunk = 1) "
                    "but the static array holds %zu; use grf_masked_linear_attention_fused with a workspace", one, kStaticScratchBytes);
    int64_t step = 1;
    if (slices > 1) {
        const size_t per_slice = grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, 2) - one;
        step = 1 + static_cast<int64_t>((kStaticScratchBytes - one) / (per_slice > 0 ? per_slice : 1));
        if (step > slices) step = slices;
        while (step > 1 && grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, static_cast<int32_t>(step)) > kStaticScratchBytes) --step;
    }
    unsigned char* ws = nullptr;
    if (grf_status st = static_scratch(&ws)) return st;
    return fused_impl(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, step, ws, static_cast<hipStream_t>(hip_stream),
                      out, num_opt, den_opt);
}
