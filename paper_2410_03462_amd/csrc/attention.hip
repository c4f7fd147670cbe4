// GRF-masked linear attention (Eq. 7; Alg. 1 steps 3-5) on gfx950.
//
//   transpose   Phi_hat CSR -> column lists (who contributes to bucket l), rows ascending
//   buckets     S_l = sum_j Phi_hat[j,l] phi(k_j) v_j^T,  z_l = sum_j Phi_hat[j,l] phi(k_j)
//               one wavefront per (slice, l); the (d x r_l)(r_l x d) contraction runs on fp32 MFMA
//   gather      num_i = sum_l Phi_hat[i,l] phi(q_i)^T S_l, den_i likewise with z_l; out = num/den
//               one wavefront per (slice, i); streams one contiguous bucket record per entry
//
// A bucket record is d*d floats of S_l (S_l[a][c] at a*d + c, a = feature index of phi(k)) followed
// by d floats of z_l, so the gather reads one contiguous run per entry of Phi_hat.
#include <atomic>

#include "attention_common.hpp"

namespace grf {

// ------------------------------------------------------------------------------------ transpose
// Entries per column; the arrival index of every entry within its column (what the atomic returns) is kept,
// so that the scatter below needs no second round of atomics.
__global__ __launch_bounds__(256) void column_histogram_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                               long long nnz, int32_t n,
                                                               int32_t* __restrict__ count, int32_t* __restrict__ arrival)
{
    const long long e = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    if (e >= row_ptr[n]) { arrival[e] = -1; return; }      // nnz may be an upper bound: the rows end at row_ptr[n]
    const int32_t c = col[e];
    arrival[e] = static_cast<uint32_t>(c) < static_cast<uint32_t>(n) ? atomicAdd(&count[c], 1) : -1;
}

// One wavefront per row: (row, entry index) of every entry goes to slot col_ptr[c] + arrival.  The order inside
// a segment depends on atomic arrival and is fixed afterwards by column_sort_kernel.
__global__ __launch_bounds__(256) void column_scatter_kernel(const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                             long long nnz, int32_t n, const int32_t* __restrict__ col_ptr,
                                                             const int32_t* __restrict__ arrival, int32_t* __restrict__ u_row,
                                                             int32_t* __restrict__ u_src)
{
    const long long row = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (row >= n) return;
    const long long beg = max(static_cast<long long>(row_ptr[row]), 0ll);      // a malformed row_ptr must not cost a long empty loop
    long long end = row_ptr[row + 1];
    if (end > nnz) end = nnz;
    for (long long e = beg + lane_id(); e < end; e += kWave) {
        const int32_t c = col[e];
        const int32_t k = arrival[e];
        if (static_cast<uint32_t>(c) >= static_cast<uint32_t>(n) || k < 0) continue;
        const int32_t slot = col_ptr[c] + k;
        if (slot >= col_ptr[c + 1]) continue;   // only with overlapping rows in a malformed row_ptr
        u_row[slot] = static_cast<int32_t>(row);
        u_src[slot] = static_cast<int32_t>(e);
    }
}

// One thread per position of the column lists: order each segment by row index (rows are distinct within a
// column) by counting, so that the buckets are summed in a fixed order.  A position finds its column by
// bisection of col_ptr and scans that column's segment; lanes of a wavefront mostly share the column, so the
// scan reads are broadcasts.  The work is quadratic in a column's length but spread over as many wavefronts as
// the column has blocks of 64 entries, so one very long column (a hub node) does not serialise the launch.
__global__ __launch_bounds__(256) void column_sort_kernel(const int32_t* __restrict__ col_ptr, int32_t n, int32_t nnz,
                                                          const int32_t* __restrict__ u_row, const int32_t* __restrict__ u_src,
                                                          int32_t* __restrict__ s_row, int32_t* __restrict__ s_src,
                                                          int32_t* __restrict__ csr_to_csc, int32_t* __restrict__ span)
{
    const long long p = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= nnz || p >= col_ptr[n]) return;      // nnz may be an upper bound: the lists end at col_ptr[n]
    int32_t lo = 0, hi = n;                 // col_ptr[lo] <= p < col_ptr[hi]
    while (hi - lo > 1) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (col_ptr[mid] <= p) lo = mid; else hi = mid;
    }
    const int32_t beg = col_ptr[lo];
    const int32_t len = col_ptr[lo + 1] - beg;
    const int32_t key = u_row[p];
    int rank = 0;
    for (int s2 = 0; s2 < len; ++s2) rank += static_cast<int>(u_row[beg + s2] < key);
    const int32_t src = u_src[p];
    // Slots that a malformed Phi_hat (overlapping rows) left unset hold arbitrary bits: whatever is
    // written downstream is a valid index, so the kernels that follow need no guards.
    const bool ok = static_cast<uint32_t>(key) < static_cast<uint32_t>(n) && static_cast<uint32_t>(src) < static_cast<uint32_t>(nnz) && rank < len;
    if (ok) {
        s_row[beg + rank] = key;
        s_src[beg + rank] = src;
        csr_to_csc[src] = beg + rank;
        span[beg + rank] = rank | (min(len, 255) << 8);
    }
}

// Value planes in column-list order: s_val[h][pos] = val[h][s_src[pos]].
__global__ __launch_bounds__(256) void column_values_kernel(const int32_t* __restrict__ col_ptr, int32_t n,
                                                            const int32_t* __restrict__ s_src, long long nnz, int n_f,
                                                            const float* __restrict__ val, long long val_stride,
                                                            float* __restrict__ s_val)
{
    const long long pos = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (pos >= nnz || pos >= col_ptr[n]) return;
    const int32_t src = s_src[pos];
    for (int h = 0; h < n_f; ++h) s_val[h * nnz + pos] = val[h * val_stride + src];
}

// Longest list among those of at most kGramPackMax entries (0 if there is none): it sets the width of the plan's windows.
__global__ __launch_bounds__(256) void short_list_max_kernel(const int32_t* __restrict__ col_ptr, int32_t n, int32_t* __restrict__ counts)
{
    const long long l = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    int32_t len = 0;
    if (l < n) {
        len = col_ptr[l + 1] - col_ptr[l];
        if (len > kGramPackMax) len = 0;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) len = max(len, __shfl_xor(len, off, kWave));
    if (lane_id() == 0 && len > 0) atomicMax(counts + kPlanMaxShort, len);
}

// Work items of the short-list kernels and the list of the long buckets.  With L the longest list of at most
// kGramPackMax entries, the entry sequence is cut into windows of W = kGramTile + 1 - L entries (at least kGramWindow): the
// lists of at most kGramPackMax entries that start inside one window span at most W - 1 + L = kGramTile entries, and
// the shorter the graph's lists, the wider the windows and the fuller the runs.  One thread per window walks the
// buckets that start in it: consecutive short lists form a run; a list of up to kGramMaxList entries is a run by itself;
// a longer one goes to the list of long buckets.  Runs and long buckets are appended with one atomic per wavefront and
// round (a window yields one run and at most one other bucket in nearly all cases); their order is not fixed and nothing
// depends on it.
__global__ __launch_bounds__(256) void window_plan_kernel(const int32_t* __restrict__ col_ptr, int32_t n, long long n_windows,
                                                          int2* __restrict__ items, long long item_capacity,
                                                          int32_t* __restrict__ long_list, int32_t* __restrict__ counts)
{
    const long long w = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int32_t width = min(max(kGramTile + 1 - counts[kPlanMaxShort], kGramWindow), kGramTile);
    // first bucket in [0, n) whose list starts at or after entry x (n if none)
    auto first_from = [&](long long x) {
        int32_t lo = 0, hi = n;
        while (lo < hi) {
            const int32_t mid = lo + (hi - lo) / 2;
            if (col_ptr[mid] >= x) hi = mid; else lo = mid + 1;
        }
        return lo;
    };
    auto append = [&](bool have, int32_t* counter) -> int32_t {
        const unsigned long long mask = __ballot(have);
        int32_t base = 0;
        if (lane_id() == 0 && mask != 0ull) base = atomicAdd(counter, __popcll(mask));
        base = __shfl(base, 0, kWave);
        return base + prefix_popcount(mask);
    };
    int32_t l = 0, lb = 0;
    if (w < n_windows && w * width < col_ptr[n]) { l = first_from(w * width); lb = first_from((w + 1) * width); }
    while (__ballot(l < lb) != 0ull) {      // the same number of rounds for the whole wavefront
        int2 run = make_int2(0, 0);
        int32_t long_bucket = -1;
        while (l < lb) {      // short lists from l on
            const int32_t b = col_ptr[l], e = col_ptr[l + 1];
            if (e - b > kGramPackMax) break;
            if (e > b) { if (run.y == run.x) run.x = b; run.y = e; }
            ++l;
        }
        if (l < lb) {         // the bucket that ended the run: to the long ones at once, else a run of its own (next round if one is pending)
            const int32_t b = col_ptr[l], e = col_ptr[l + 1];
            if (e - b > kGramMaxList) { long_bucket = l; ++l; }
            else if (run.y == run.x) { run = make_int2(b, e); ++l; }
        }
        const bool has_run = run.y > run.x && run.y - run.x <= kGramTile;
        const int32_t at_run = append(has_run, counts + kPlanItems);
        if (has_run && at_run < item_capacity) items[at_run] = run;
        const int32_t at_long = append(long_bucket >= 0, counts + kPlanLong);
        if (long_bucket >= 0 && at_long < n) long_list[at_long] = long_bucket;
    }
}

// ------------------------------------------------------------------------------------ buckets
// v_mfma_f32_32x32x2_f32: D(32x32) += A(32x2) B(2x32).  Lane L supplies A[L%32][L/32] and
// B[L/32][L%32]; accumulator register r of lane L holds D[8*(r/4) + 4*(L/32) + r%4][L%32].
// The two halves of the wavefront therefore carry two different contributors j (the k index),
// lane%32 walks along a row of phi(K) (A operand) and of V (B operand): no transposes, no LDS.
template <int D, typename T, bool WIDE>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2))) void buckets_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                      long long n, int H, int n_f,
                                                      const int32_t* __restrict__ col_ptr, const int32_t* __restrict__ csc_row,
                                                      const float* __restrict__ csc_val,
                                                      int fmap, long long bh_first, long long n_waves, int32_t nnz,
                                                      float* __restrict__ buckets)
{
    constexpr int T2 = D / 32;
    constexpr long long REC = static_cast<long long>(D) * D + D;
    const uint32_t wave = blockIdx.x;          // one wavefront per workgroup: column lists differ in length
    if (wave >= n_waves) return;
    const uint32_t slice32 = wave / static_cast<uint32_t>(n);      // slice index inside this launch; B*H*n < 2^31, and a
    const long long slice = slice32;                               // 32-bit division is a fraction of a 64-bit one
    const long long l = wave - slice32 * static_cast<uint32_t>(n);
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (static_cast<uint32_t>(bh) % static_cast<uint32_t>(H)) : 0u;
    const T* Kb = K + bh * n * D;
    const T* Vb = V + bh * n * D;
    const float* vals = csc_val + plane * nnz;

    const int lane = lane_id();
    const int half = lane >> 5;
    const int li = lane & 31;

    floatx16 acc[T2][T2];
    float zacc[T2];
    const int32_t beg = col_ptr[l], end = col_ptr[l + 1];
    const ListBlock first = load_list_block<false>(csc_row, vals, nullptr, beg, end);
    with_feature_map(fmap, [&](auto fm) {
        bucket_first_contraction<D, T, T, false, true, kExtraSumA, decltype(fm)::value, WIDE>(Kb, Vb, csc_row, vals, nullptr, beg, end, first, acc, zacc);
    });

    float* rec = buckets + (slice * n + l) * REC;
#pragma unroll
    for (int a = 0; a < T2; ++a)
#pragma unroll
        for (int c = 0; c < T2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * a + 8 * (r / 4) + 4 * half + (r % 4);
                rec[row * D + 32 * c + li] = acc[a][c][r];
            }
#pragma unroll
    for (int a = 0; a < T2; ++a) {
        const float zt = zacc[a] + __shfl_xor(zacc[a], 32, kWave);
        if (half == 0) rec[D * D + 32 * a + li] = zt;
    }
}

// ------------------------------------------------------------------------------------ gather
// One wavefront per (slice, row i).  A record is read with 16-byte loads: lane L covers columns
// 4*(L % (D/4)) .. +3 of row  j*(256/D) + L/(D/4)  for load j; the weight Phi_hat[i,l] * phi(q_i)[row]
// is applied on the fly, so only four accumulators per lane are live and the reduction over the
// D/ (256/D) row groups happens once per output row.
template <int D, typename T>
__global__ __launch_bounds__(256) void gather_kernel(const T* __restrict__ Q, long long n, int H, int n_f, long long val_stride,
                                                     const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                                                     const float* __restrict__ phi_val, int fmap,
                                                     const float* __restrict__ buckets, long long bh_first, long long n_waves,
                                                     int32_t nnz, int spread_xcds,
                                                     float* __restrict__ out, float* __restrict__ num_opt, float* __restrict__ den_opt)
{
    constexpr int LPR = D / 4;            // lanes per record row
    constexpr int RPL = kWave / LPR;      // record rows per 1 KB load
    constexpr int NL = D / RPL;           // loads per record
    constexpr long long REC = static_cast<long long>(D) * D + D;
    // Workgroups go to the eight XCDs round-robin by id.  spread_xcds: each XCD takes a contiguous eighth of all
    // (slice, row) pairs, so that a slice's records pass through one L2 instead of all eight (right when eight
    // slices' records fit the Infinity Cache; with larger slices the wider footprint in flight costs more in address
    // translation than the L2 saves).
    const long long block = spread_xcds ? xcd_contiguous_block(blockIdx.x, gridDim.x) : static_cast<long long>(blockIdx.x);
    const long long wave = block * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (wave >= n_waves) return;
    const long long slice = wave / n;
    const long long i = wave - slice * n;
    const long long bh = bh_first + slice;
    const long long plane = n_f > 1 ? (bh % H) : 0;
    const float* vals = phi_val + plane * val_stride;
    const T* q = Q + (bh * n + i) * D;
    const float* slice_buckets = buckets + slice * n * REC;

    const int lane = lane_id();
    const int sub = lane / LPR;
    const int cg = lane % LPR;

    float fq[NL];
#pragma unroll
    for (int j = 0; j < NL; ++j) fq[j] = feature(to_float(q[j * RPL + sub]), fmap);
    const float fq_lane = lane < D ? feature(to_float(q[lane < D ? lane : 0]), fmap) : 0.0f;

    float acc0 = 0.0f, acc1 = 0.0f, acc2 = 0.0f, acc3 = 0.0f, zacc = 0.0f;

    const int32_t beg = max(row_ptr[i], 0);
    const int32_t end = min(row_ptr[i + 1], nnz);
    for (int32_t chunk = beg; chunk < end; chunk += kWave) {
        const int32_t e = chunk + lane;
        int32_t c_reg = 0;
        float w_reg = 0.0f;
        if (e < end) { c_reg = col[e]; w_reg = vals[e]; }
        const int cnt = min(kWave, end - chunk);
        for (int t = 0; t < cnt; ++t) {
            const int32_t c = __builtin_amdgcn_readlane(c_reg, t);
            const float w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w_reg), t));
            if (static_cast<uint32_t>(c) >= static_cast<uint32_t>(n)) continue;
            const float* rec = slice_buckets + static_cast<long long>(c) * REC;
            const float4* rec4 = reinterpret_cast<const float4*>(rec) + lane;
            float4 v[NL];
#pragma unroll
            for (int j = 0; j < NL; ++j) v[j] = rec4[j * kWave];
            const float zv = lane < D ? rec[D * D + (lane < D ? lane : 0)] : 0.0f;
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                const float wq = w * fq[j];
                acc0 = fmaf(wq, v[j].x, acc0);
                acc1 = fmaf(wq, v[j].y, acc1);
                acc2 = fmaf(wq, v[j].z, acc2);
                acc3 = fmaf(wq, v[j].w, acc3);
            }
            zacc = fmaf(w, zv, zacc);
        }
    }

#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
        acc0 += __shfl_xor(acc0, off, kWave);
        acc1 += __shfl_xor(acc1, off, kWave);
        acc2 += __shfl_xor(acc2, off, kWave);
        acc3 += __shfl_xor(acc3, off, kWave);
    }
    const float den = wave_sum(fq_lane * zacc);

    if (sub == 0) {
        const long long o = (bh * n + i) * D + 4 * cg;
        *reinterpret_cast<float4*>(out + o) = make_float4(acc0 / den, acc1 / den, acc2 / den, acc3 / den);
        if (num_opt != nullptr) *reinterpret_cast<float4*>(num_opt + o) = make_float4(acc0, acc1, acc2, acc3);
    }
    if (lane == 0 && den_opt != nullptr) den_opt[bh * n + i] = den;
}

// ------------------------------------------------------------------------------------ host side
Transposed carve_transposed(unsigned char* ws, int64_t n, int64_t nnz, int32_t n_f)
{
    Transposed t;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = ws ? ws + off : nullptr; off += align_up(bytes); return p; };
    const size_t entries = static_cast<size_t>(nnz > 0 ? nnz : 1);
    t.col_ptr = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(n + 1)));
    t.u_row = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.u_src = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.s_row = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.s_src = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.csr_to_csc = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.arrival = t.csr_to_csc;      // the arrival indices are dead before the positions are written
    t.s_val = reinterpret_cast<float*>(take(sizeof(float) * entries * static_cast<size_t>(n_f > 0 ? n_f : 1)));
    t.span = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * entries));
    t.n_windows = static_cast<long long>((entries + kGramWindow - 1) / kGramWindow);
    t.item_capacity = static_cast<long long>(nnz < n ? (nnz > 0 ? nnz : 1) : (n > 0 ? n : 1));      // a run holds at least one non-empty list
    t.items = reinterpret_cast<int2*>(take(sizeof(int2) * static_cast<size_t>(t.item_capacity)));
    t.long_list = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * static_cast<size_t>(n > 0 ? n : 1)));
    t.plan_counts = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * kPlanCounters));
    t.total = reinterpret_cast<long long*>(take(sizeof(long long)));
    t.bytes = off;
    return t;
}

grf_status transpose(const grf_phi* phi, int64_t nnz, int32_t n_f, const Transposed& t, hipStream_t stream)
{
    const int64_t n = phi->n;
    if (grf_status st = fill_i32(t.col_ptr, n + 1, 0, stream)) return st;
    if (grf_status st = fill_i32(t.plan_counts, kPlanCounters, 0, stream)) return st;
    if (nnz > 0) {
        if (grf_status st = fill_i32(t.s_row, nnz, 0, stream)) return st;
        if (grf_status st = fill_i32(t.s_src, nnz, 0, stream)) return st;
        hipLaunchKernelGGL(column_histogram_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(phi->row_ptr), static_cast<const int32_t*>(phi->col),
                           static_cast<long long>(nnz), static_cast<int32_t>(n), t.col_ptr, t.arrival);
        GRF_LAUNCH_CHECK("column_histogram_kernel");
    }
    if (grf_status st = exclusive_scan_inplace(t.col_ptr, n, t.total, stream)) return st;
    if (nnz > 0) {
        hipLaunchKernelGGL(column_scatter_kernel, dim3(blocks_for(n, 4)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(phi->row_ptr), static_cast<const int32_t*>(phi->col),
                           static_cast<long long>(nnz), static_cast<int32_t>(n), static_cast<const int32_t*>(t.col_ptr),
                           static_cast<const int32_t*>(t.arrival), t.u_row, t.u_src);
        GRF_LAUNCH_CHECK("column_scatter_kernel");
        // entries that a malformed Phi_hat never reaches must not point anywhere
        if (grf_status st = fill_i32(t.csr_to_csc, nnz, -1, stream)) return st;
        hipLaunchKernelGGL(column_sort_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(t.col_ptr), static_cast<int32_t>(n), static_cast<int32_t>(nnz),
                           static_cast<const int32_t*>(t.u_row), static_cast<const int32_t*>(t.u_src), t.s_row, t.s_src,
                           t.csr_to_csc, t.span);
        GRF_LAUNCH_CHECK("column_sort_kernel");
        hipLaunchKernelGGL(short_list_max_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(t.col_ptr), static_cast<int32_t>(n), t.plan_counts);
        GRF_LAUNCH_CHECK("short_list_max_kernel");
        hipLaunchKernelGGL(window_plan_kernel, dim3(blocks_for(t.n_windows, 256)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(t.col_ptr), static_cast<int32_t>(n), t.n_windows, t.items, t.item_capacity,
                           t.long_list, t.plan_counts);
        GRF_LAUNCH_CHECK("window_plan_kernel");
        hipLaunchKernelGGL(column_values_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, stream,
                           static_cast<const int32_t*>(t.col_ptr), static_cast<int32_t>(n),
                           static_cast<const int32_t*>(t.s_src), static_cast<long long>(nnz), static_cast<int>(n_f),
                           static_cast<const float*>(phi->val), static_cast<long long>(phi->capacity), t.s_val);
        GRF_LAUNCH_CHECK("column_values_kernel");
    }
    return GRF_OK;
}

grf_status check_problem(const void* a, const void* b, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                         const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map)
{
    if (B < 0 || H < 0 || n < 0) return fail(GRF_EINVAL, "B=%lld, H=%lld, n=%lld must be >= 0", (long long)B, (long long)H, (long long)n);
    // one wavefront (or workgroup) per (slice, node) in the launches that follow; tensors of 2^31 rows would
    // not fit the device anyway
    if ((B > 0 && H > 2147483647ll / B) || (n > 0 && B * H > 2147483647ll / n))
        return fail(GRF_EUNSUPPORTED, "B*H*n = %lld*%lld*%lld must be < 2^31", (long long)B, (long long)H, (long long)n);
    if (dtype != GRF_DTYPE_F32 && dtype != GRF_DTYPE_BF16) return fail(GRF_EINVAL, "dtype=%d is neither GRF_DTYPE_F32 nor GRF_DTYPE_BF16", dtype);
    if (feature_map != GRF_PHI_RELU && feature_map != GRF_PHI_IDENTITY && feature_map != GRF_PHI_ELU1) return fail(GRF_EINVAL, "feature_map=%d is unknown", feature_map);
    if (d != 32 && d != 64) return fail(GRF_EUNSUPPORTED, "head dimension d=%d is not supported (32 or 64)", d);
    if (phi == nullptr) return fail(GRF_EINVAL, "phi is NULL");
    if (phi->n != n) return fail(GRF_EINVAL, "phi->n=%lld differs from n=%lld", (long long)phi->n, (long long)n);
    if (nnz < 0 || nnz > phi->capacity) return fail(GRF_EINVAL, "nnz=%lld must lie in [0, phi->capacity=%lld]", (long long)nnz, (long long)phi->capacity);
    if (nnz >= 2147483647ll - 256 || n >= 2147483647ll - 256) return fail(GRF_EUNSUPPORTED, "n and nnz must be < 2^31 - 257");
    if (n_f != 1 && n_f != H) return fail(GRF_EINVAL, "n_f=%d must be 1 or H=%lld", n_f, (long long)H);
    if (phi->row_ptr == nullptr || (nnz > 0 && (phi->col == nullptr || phi->val == nullptr))) return fail(GRF_EINVAL, "phi arrays are NULL");
    if (B * H * n > 0 && (a == nullptr || b == nullptr)) return fail(GRF_EINVAL, "an input tensor is NULL");
    return GRF_OK;
}

namespace {
std::atomic<int> g_force_wide_offsets{0};
}

bool wide_offsets(int64_t n, int32_t d)
{
    return g_force_wide_offsets.load(std::memory_order_relaxed) != 0 || n * static_cast<int64_t>(d) * 4 > 0xffffffffll;
}

unsigned resident_wave_grid(const void* kernel, long long items)
{
    int device = 0, units = 0, per_unit = 0;
    if (hipGetDevice(&device) != hipSuccess || hipDeviceGetAttribute(&units, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_unit, kernel, kWave, 0) != hipSuccess || units < 1 || per_unit < 1) {
        units = 256; per_unit = 8;       // an MI355X with two wavefronts per SIMD
    }
    const long long resident = static_cast<long long>(units) * per_unit;
    return static_cast<unsigned>(items < resident ? (items > 0 ? items : 1) : resident);
}

grf_status check_workspace(const void* workspace, size_t have, size_t need)
{
    if (workspace == nullptr || have < need || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return fail(GRF_EWORKSPACE, "workspace must be non-NULL, 256-byte aligned and >= %zu bytes (got %zu)", need, have);
    return GRF_OK;
}

namespace {

template <int D, typename T>
grf_status launch_buckets(const void* K, const void* V, int64_t n, int64_t H, int32_t n_f,
                          int64_t nnz, const Transposed& t, int fmap, int64_t bh_first, int64_t n_slices, float* buckets,
                          hipStream_t stream)
{
    const long long waves = static_cast<long long>(n_slices) * n;
    if (waves == 0) return GRF_OK;
    auto launch = [&](auto wide) {
        hipLaunchKernelGGL((buckets_kernel<D, T, decltype(wide)::value>), dim3(blocks_for(waves, 1)), dim3(kWave), 0, stream,
                           static_cast<const T*>(K), static_cast<const T*>(V), static_cast<long long>(n), static_cast<int>(H),
                           static_cast<int>(n_f),
                           static_cast<const int32_t*>(t.col_ptr), static_cast<const int32_t*>(t.s_row),
                           static_cast<const float*>(t.s_val), fmap,
                           static_cast<long long>(bh_first), waves, static_cast<int32_t>(nnz), buckets);
    };
    if (wide_offsets(n, D)) launch(std::true_type{}); else launch(std::false_type{});
    GRF_LAUNCH_CHECK("buckets_kernel");
    return GRF_OK;
}

template <int D, typename T>
grf_status launch_gather(const void* Q, int64_t n, int64_t H, int32_t n_f, const grf_phi* phi, int64_t nnz, int fmap,
                         const float* buckets, int64_t bh_first, int64_t n_slices,
                         float* out, float* num_opt, float* den_opt, hipStream_t stream)
{
    const long long waves = static_cast<long long>(n_slices) * n;
    if (waves == 0) return GRF_OK;
    const int spread = 8ll * n * (D * D + D) * 4 <= (256ll << 20) ? 1 : 0;      // see the kernel
    hipLaunchKernelGGL((gather_kernel<D, T>), dim3(blocks_for(waves, 4)), dim3(256), 0, stream,
                       static_cast<const T*>(Q), static_cast<long long>(n), static_cast<int>(H), static_cast<int>(n_f),
                       static_cast<long long>(phi->capacity), static_cast<const int32_t*>(phi->row_ptr),
                       static_cast<const int32_t*>(phi->col), static_cast<const float*>(phi->val), fmap, buckets,
                       static_cast<long long>(bh_first), waves, static_cast<int32_t>(nnz), spread, out, num_opt, den_opt);
    GRF_LAUNCH_CHECK("gather_kernel");
    return GRF_OK;
}

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" void grf_debug_force_wide_offsets(int32_t on)
{
    g_force_wide_offsets.store(on != 0 ? 1 : 0, std::memory_order_relaxed);
}

extern "C" int64_t grf_bucket_record_floats(int32_t d)
{
    if (d != 32 && d != 64) return -1;
    return static_cast<int64_t>(d) * d + d;
}

extern "C" size_t grf_buckets_workspace_bytes(int64_t n, int64_t nnz, int32_t n_f)
{
    if (n < 0 || nnz < 0 || n_f < 1) return 0;
    return carve_transposed(nullptr, n, nnz, n_f).bytes;
}

extern "C" size_t grf_attention_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk)
{
    if (B < 0 || H < 0 || n < 0 || nnz < 0 || n_f < 1 || (d != 32 && d != 64)) return 0;
    int64_t slices = B * H;
    if (bh_chunk > 0 && bh_chunk < slices) slices = bh_chunk;
    const size_t bucket_bytes = sizeof(float) * static_cast<size_t>(slices) * static_cast<size_t>(n) * static_cast<size_t>(grf_bucket_record_floats(d));
    return carve_transposed(nullptr, n, nnz, n_f).bytes + align_up(bucket_bytes);
}

namespace grf {

grf_status check_phi(const grf_phi* phi, int64_t nnz, int32_t n_f)
{
    if (phi == nullptr) return fail(GRF_EINVAL, "phi is NULL");
    if (phi->n < 0) return fail(GRF_EINVAL, "phi->n=%lld must be >= 0", (long long)phi->n);
    if (nnz < 0 || nnz > phi->capacity) return fail(GRF_EINVAL, "nnz=%lld must lie in [0, phi->capacity=%lld]", (long long)nnz, (long long)phi->capacity);
    if (nnz >= 2147483647ll - 256 || phi->n >= 2147483647ll - 256) return fail(GRF_EUNSUPPORTED, "n and nnz must be < 2^31 - 257");
    if (n_f < 1) return fail(GRF_EINVAL, "n_f=%d must be >= 1", n_f);
    if (phi->row_ptr == nullptr || (nnz > 0 && (phi->col == nullptr || phi->val == nullptr))) return fail(GRF_EINVAL, "phi arrays are NULL");
    return GRF_OK;
}

grf_status prepared_lists(const void* prepared, size_t prepared_bytes, int64_t n, int64_t nnz, int32_t n_f, Transposed* t)
{
    const size_t need = carve_transposed(nullptr, n, nnz, n_f).bytes;
    if (prepared == nullptr || prepared_bytes < need || (reinterpret_cast<uintptr_t>(prepared) % kAlign) != 0)
        return fail(GRF_EWORKSPACE, "prepared must be non-NULL, 256-byte aligned and >= grf_phi_prepare_bytes() = %zu bytes (got %zu)", need, prepared_bytes);
    *t = carve_transposed(static_cast<unsigned char*>(const_cast<void*>(prepared)), n, nnz, n_f);
    return GRF_OK;
}

grf_status launch_column_values(const grf_phi* phi, int64_t nnz, int32_t n_f, const Transposed& t, hipStream_t stream)
{
    if (nnz <= 0) return GRF_OK;
    hipLaunchKernelGGL(column_values_kernel, dim3(blocks_for(nnz, 256)), dim3(256), 0, stream,
                       static_cast<const int32_t*>(t.col_ptr), static_cast<int32_t>(phi->n),
                       static_cast<const int32_t*>(t.s_src), static_cast<long long>(nnz), static_cast<int>(n_f),
                       static_cast<const float*>(phi->val), static_cast<long long>(phi->capacity), t.s_val);
    GRF_LAUNCH_CHECK("column_values_kernel");
    return GRF_OK;
}

namespace {

grf_status form_buckets_impl(const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                             int64_t nnz, int32_t n_f, int32_t feature_map, const Transposed& t, hipStream_t stream, float* buckets)
{
    grf_status st = GRF_OK;
    GRF_DISPATCH(d, dtype, (st = launch_buckets<D_, T_>(K, V, n, H, n_f, nnz, t, feature_map, 0, B * H, buckets, stream)));
    return st;
}

grf_status attention_impl(const void* Q, const void* K, const void* V, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                          const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map, int32_t bh_chunk,
                          const Transposed& t, float* buckets, hipStream_t stream, float* out, float* num_opt, float* den_opt)
{
    const int fmap = feature_map;
    const int64_t slices = B * H;
    const int64_t step = (bh_chunk > 0 && bh_chunk < slices) ? bh_chunk : slices;
    for (int64_t first = 0; first < slices; first += step) {
        const int64_t count = (slices - first < step) ? (slices - first) : step;
        grf_status st = GRF_OK;
        GRF_DISPATCH(d, dtype, (st = launch_buckets<D_, T_>(K, V, n, H, n_f, nnz, t, fmap, first, count, buckets, stream)));
        if (st != GRF_OK) return st;
        GRF_DISPATCH(d, dtype, (st = launch_gather<D_, T_>(Q, n, H, n_f, phi, nnz, fmap, buckets, first, count, out, num_opt, den_opt, stream)));
        if (st != GRF_OK) return st;
    }
    return GRF_OK;
}

size_t bucket_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int32_t bh_chunk)
{
    int64_t slices = B * H;
    if (bh_chunk > 0 && bh_chunk < slices) slices = bh_chunk;
    return align_up(sizeof(float) * static_cast<size_t>(slices) * static_cast<size_t>(n) * static_cast<size_t>(grf_bucket_record_floats(d)));
}

}  // namespace
}  // namespace grf

extern "C" size_t grf_phi_prepare_bytes(int64_t n, int64_t nnz, int32_t n_f)
{
    return grf_buckets_workspace_bytes(n, nnz, n_f);
}

extern "C" grf_status grf_phi_prepare(const grf_phi* phi, int64_t nnz, int32_t n_f, void* prepared, size_t prepared_bytes, void* hip_stream)
{
    if (grf_status st = check_phi(phi, nnz, n_f)) return st;
    Transposed t;
    if (grf_status st = prepared_lists(prepared, prepared_bytes, phi->n, nnz, n_f, &t)) return st;
    return transpose(phi, nnz, n_f, t, static_cast<hipStream_t>(hip_stream));
}

extern "C" grf_status grf_phi_prepare_values(const grf_phi* phi, int64_t nnz, int32_t n_f, void* prepared, size_t prepared_bytes, void* hip_stream)
{
    if (grf_status st = check_phi(phi, nnz, n_f)) return st;
    Transposed t;
    if (grf_status st = prepared_lists(prepared, prepared_bytes, phi->n, nnz, n_f, &t)) return st;
    return launch_column_values(phi, nnz, n_f, t, static_cast<hipStream_t>(hip_stream));
}

extern "C" grf_status grf_form_buckets(const void* K, const void* V, int32_t dtype,
                                       int64_t B, int64_t H, int64_t n, int32_t d,
                                       const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                       void* workspace, size_t workspace_bytes, void* hip_stream, float* buckets)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && buckets == nullptr) return fail(GRF_EINVAL, "buckets is NULL");
    if (grf_status st = check_workspace(workspace, workspace_bytes, grf_buckets_workspace_bytes(n, nnz, n_f))) return st;
    if (B * H * n == 0) return GRF_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Transposed t = carve_transposed(static_cast<unsigned char*>(workspace), n, nnz, n_f);
    if (grf_status st = transpose(phi, nnz, n_f, t, stream)) return st;
    return form_buckets_impl(K, V, dtype, B, H, n, d, nnz, n_f, feature_map, t, stream, buckets);
}

extern "C" grf_status grf_form_buckets_prepared(const void* K, const void* V, int32_t dtype,
                                                int64_t B, int64_t H, int64_t n, int32_t d,
                                                const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                const void* prepared, size_t prepared_bytes, void* hip_stream, float* buckets)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && buckets == nullptr) return fail(GRF_EINVAL, "buckets is NULL");
    Transposed t;
    if (grf_status st = prepared_lists(prepared, prepared_bytes, n, nnz, n_f, &t)) return st;
    if (B * H * n == 0) return GRF_OK;
    return form_buckets_impl(K, V, dtype, B, H, n, d, nnz, n_f, feature_map, t, static_cast<hipStream_t>(hip_stream), buckets);
}

extern "C" grf_status grf_gather_buckets(const void* Q, int32_t dtype,
                                         int64_t B, int64_t H, int64_t n, int32_t d,
                                         const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                         const float* buckets, void* hip_stream,
                                         float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(Q, buckets, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && out == nullptr) return fail(GRF_EINVAL, "out is NULL");
    if (B * H * n == 0) return GRF_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int fmap = feature_map;
    grf_status st = GRF_OK;
    GRF_DISPATCH(d, dtype, (st = launch_gather<D_, T_>(Q, n, H, n_f, phi, nnz, fmap, buckets, 0, B * H, out, num_opt, den_opt, stream)));
    return st;
}

extern "C" grf_status grf_masked_linear_attention(const void* Q, const void* K, const void* V, int32_t dtype,
                                                  int64_t B, int64_t H, int64_t n, int32_t d,
                                                  const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                  int32_t bh_chunk,
                                                  void* workspace, size_t workspace_bytes, void* hip_stream,
                                                  float* out, float* num_opt, float* den_opt)
{
    if (grf_status st = check_problem(K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map)) return st;
    if (B * H * n > 0 && (Q == nullptr || out == nullptr)) return fail(GRF_EINVAL, "Q / out is NULL");
    if (grf_status st = check_workspace(workspace, workspace_bytes, grf_attention_workspace_bytes(B, H, n, d, nnz, n_f, bh_chunk))) return st;
    if (B * H * n == 0) return GRF_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Transposed t = carve_transposed(static_cast<unsigned char*>(workspace), n, nnz, n_f);
    float* buckets = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + t.bytes);
    if (grf_status st = transpose(phi, nnz, n_f, t, stream)) return st;
    return attention_impl(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, bh_chunk, t, buckets, stream, out, num_opt, den_opt);
}

extern "C" grf_status grf_masked_linear_attention_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
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
    if (grf_status st = check_workspace(workspace, workspace_bytes, bucket_bytes(B, H, n, d, bh_chunk))) return st;
    if (B * H * n == 0) return GRF_OK;
    return attention_impl(Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, bh_chunk, t, static_cast<float*>(workspace),
                          static_cast<hipStream_t>(hip_stream), out, num_opt, den_opt);
}
