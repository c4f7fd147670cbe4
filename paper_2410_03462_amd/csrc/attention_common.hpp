// Pieces shared by the attention translation units: element loads, the column lists of
// Phi_hat (who contributes to / consumes bucket l) and host-side argument checks.
#pragma once

#include <type_traits>

#include "common.hpp"

namespace grf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.bits) << 16); }

// max(x, 0) as one integer maximum of the bit pattern with 0: floats with the sign bit clear order like
// integers, all others (negative values, -0) are negative integers.  (A floating-point maximum costs a second
// instruction that quiets signalling NaNs first.)
__device__ __forceinline__ float relu(float x) { return __int_as_float(max(__float_as_int(x), 0)); }

// phi(x) for the feature-map codes of grf.h: max(x, 0), the identity, or elu(x) + 1 (x + 1 for x > 0,
// exp(x) otherwise).  `fmap` is wave-uniform.
__device__ __forceinline__ float feature(float x, int fmap)
{
    const float elu1 = x > 0.0f ? x + 1.0f : __expf(x);
    return fmap == GRF_PHI_RELU ? relu(x) : (fmap == GRF_PHI_ELU1 ? elu1 : x);
}

// The same with the code known at compile time (the MFMA kernels' inner loops).
template <int FM>
__device__ __forceinline__ float feature_ct(float x)
{
    if constexpr (FM == GRF_PHI_RELU) return relu(x);
    else if constexpr (FM == GRF_PHI_ELU1) return x > 0.0f ? x + 1.0f : __expf(x);
    else return x;
}

// Runs body(std::integral_constant<int, code>) for the wave-uniform feature-map code `fmap`, so that
// the body is compiled once per map and the map costs nothing inside it.
template <typename Body>
__device__ __forceinline__ void with_feature_map(int fmap, Body&& body)
{
    if (fmap == GRF_PHI_RELU) body(std::integral_constant<int, GRF_PHI_RELU>{});
    else if (fmap == GRF_PHI_ELU1) body(std::integral_constant<int, GRF_PHI_ELU1>{});
    else body(std::integral_constant<int, GRF_PHI_IDENTITY>{});
}

// d phi(x) / dx (ReLU: 0 at x = 0).
__device__ __forceinline__ float feature_grad(float x, int fmap)
{
    const float relu = x > 0.0f ? 1.0f : 0.0f;
    const float elu1 = x > 0.0f ? 1.0f : __expf(x);
    return fmap == GRF_PHI_RELU ? relu : (fmap == GRF_PHI_ELU1 ? elu1 : 1.0f);
}

// Sum of x over the 16 lanes of a row of the wavefront (lanes 16k .. 16k+15), left in every lane of the row: four
// row rotations (by 8, 4, 2, 1 lanes) on the vector ALU, no trip through the LDS crossbar.  Every lane adds the same
// pairs at each step, so the 16 results are one bit pattern.
template <int CTRL>
__device__ __forceinline__ float row_rotated(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}

__device__ __forceinline__ float row_sum16(float x)
{
    x += row_rotated<0x128>(x);      // row_ror:8
    x += row_rotated<0x124>(x);      // row_ror:4
    x += row_rotated<0x122>(x);      // row_ror:2
    x += row_rotated<0x121>(x);      // row_ror:1
    return x;
}

// N consecutive elements starting at p (p aligned to N elements), widened to fp32.
template <typename T, int N>
__device__ __forceinline__ void load_run(const T* __restrict__ p, float (&out)[N])
{
    if constexpr (sizeof(T) == 4) {
        if constexpr (N == 1) {
            out[0] = *reinterpret_cast<const float*>(p);
        } else if constexpr (N == 2) {
            const float2 v = *reinterpret_cast<const float2*>(p);
            out[0] = v.x; out[1] = v.y;
        } else {
#pragma unroll
            for (int k = 0; k < N / 4; ++k) {
                const float4 v = reinterpret_cast<const float4*>(p)[k];
                out[4 * k] = v.x; out[4 * k + 1] = v.y; out[4 * k + 2] = v.z; out[4 * k + 3] = v.w;
            }
        }
    } else {
        if constexpr (N == 1) {
            out[0] = __uint_as_float(static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(p)) << 16);
        } else {
            uint32_t w[N / 2];
            if constexpr (N == 2) {
                w[0] = *reinterpret_cast<const uint32_t*>(p);
            } else if constexpr (N == 4) {
                const uint2 v = *reinterpret_cast<const uint2*>(p);
                w[0] = v.x; w[1] = v.y;
            } else {
                const uint4 v = *reinterpret_cast<const uint4*>(p);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            }
#pragma unroll
            for (int k = 0; k < N / 2; ++k) {
                out[2 * k] = __uint_as_float(w[k] << 16);
                out[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
            }
        }
    }
}

// Lists of at most kGramMaxList entries are evaluated in runs of at most kGramTile consecutive entries of the column
// lists (gram_split.hpp): the lists of at most kGramPackMax entries that start inside one window of the entry sequence
// form one run (windows of at least kGramWindow entries, see window_plan_kernel), a longer one is a run by itself.
constexpr int kGramWindow = 16;
constexpr int kGramTile = 32;
constexpr int kGramPackMax = kGramTile - kGramWindow + 1;      // 17
constexpr int kGramMaxList = kGramTile;                        // longer lists go through S_l, one bucket per wavefront
enum : int { kPlanItems = 0, kPlanLong = 1, kPlanMaxShort = 2, kPlanCounters = 3 };      // device-side counts written by the plan

// Column lists of Phi_hat, carved out of the caller's workspace.
struct Transposed {
    int32_t* col_ptr;   // [n+1]
    int32_t* u_row;     // [nnz] unsorted
    int32_t* u_src;
    int32_t* s_row;     // [nnz] rows ascending inside each column
    int32_t* s_src;     // index of the entry in CSR order (addresses every value plane)
    int32_t* csr_to_csc;  // [nnz] position in the column lists of CSR entry e
    int32_t* arrival;     // [nnz] arrival index of entry e within its column while the lists are built (same memory)
    float* s_val;       // [n_f][nnz] value planes permuted into column-list order
    int32_t* span;      // [nnz] per list position: its index inside its list | min(list length, 255) << 8
    int2* items;        // [item_capacity] entry ranges of the runs of short lists, in no particular order (see gram_split.hpp)
    int32_t* long_list; // [n] the buckets whose lists are longer than kGramMaxList, in no particular order
    int32_t* plan_counts;   // [kPlanCounters] how many of each, on the device
    long long n_windows, item_capacity;
    long long* total;
    size_t bytes;
};

Transposed carve_transposed(unsigned char* ws, int64_t n, int64_t nnz, int32_t n_f);
grf_status transpose(const grf_phi* phi, int64_t nnz, int32_t n_f, const Transposed& t, hipStream_t stream);
grf_status check_problem(const void* a, const void* b, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                         const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map);
grf_status check_workspace(const void* workspace, size_t have, size_t need);
// The column lists inside a buffer that grf_phi_prepare filled (checked for size and alignment only).
grf_status prepared_lists(const void* prepared, size_t prepared_bytes, int64_t n, int64_t nnz, int32_t n_f, Transposed* t);

// Shared by the backward entry points (defined with the symmetric backward pass).
// g' per row: G[r][:] = d_out / den and gd[r] = -(d_out . out) / den for rows first_row .. first_row + n_rows - 1.
grf_status launch_backward_seed(int32_t d, const float* out, const float* den, const float* d_out, long long first_row,
                                long long n_rows, float* G, float* gd, hipStream_t stream);
// dphi_val[h][e] (+)= sum over the slices of a chunk that use plane h of term_a[s][e] (+ term_b[s][e] unless NULL)
// for the entries of the rows, 0 for e in [phi->row_ptr[n], nnz).
grf_status launch_dphi_accumulate(int64_t nnz, int32_t n_f, int64_t H, int64_t bh_first, int64_t n_slices,
                                  const float* term_a, const float* term_b, const grf_phi* phi, float* dphi_val,
                                  hipStream_t stream);

// Workgroups are handed to the eight XCDs round-robin by id, and each XCD has an L2 of its own.
// This maps a workgroup id to a logical index such that every XCD works through one contiguous
// range of logical indices (ids congruent mod 8 become neighbours), so that work items that are
// adjacent in the logical order share an L2.
__device__ __forceinline__ long long xcd_contiguous_block(unsigned block, unsigned n_blocks)
{
    constexpr unsigned kXcds = 8;
    const unsigned q = n_blocks / kXcds, rem = n_blocks % kXcds;
    const unsigned x = block % kXcds, k = block / kXcds;
    return static_cast<long long>(x) * q + (x < rem ? x : rem) + k;
}

// Address of element `elem` of row `row` of a [rows][D] tensor whose slice starts at `base` (wave-uniform).
// Unless WIDE, the byte offset is formed in 32 bits, which lets the load take the slice base from scalar registers
// and one vector register of offset (one vector instruction per row instead of three 64-bit ones); the host
// selects WIDE when a slice spans 4 GiB or more.
template <int D, typename T, bool WIDE>
__device__ __forceinline__ const T* row_elem_ptr(const T* __restrict__ base, uint32_t row, int elem)
{
    if constexpr (WIDE) {
        return base + (static_cast<size_t>(row) * D + elem);
    } else {
        const uint32_t off = row * static_cast<uint32_t>(D * sizeof(T)) + static_cast<uint32_t>(elem) * static_cast<uint32_t>(sizeof(T));
        return reinterpret_cast<const T*>(reinterpret_cast<const char*>(base) + off);
    }
}

// The T2 = D/32 elements of row j that MFMA row/column `li` of the tiles stands for, widened to
// fp32: element 32*t + li of the row, or, INTERLEAVED, element T2*li + t, so that a lane's
// operands are adjacent in memory (one 8-byte load at d = 64 in fp32).
template <int D, typename T, bool INTERLEAVED, bool WIDE>
__device__ __forceinline__ void load_operand_elems(const T* __restrict__ base, uint32_t j, int li, float (&x)[D / 32])
{
    constexpr int T2 = D / 32;
    if constexpr (INTERLEAVED) {
        const T* p = row_elem_ptr<D, T, WIDE>(base, j, T2 * li);
        if constexpr (sizeof(T) == 4 && T2 == 2) {
            const float2 v = *reinterpret_cast<const float2*>(p);
            x[0] = v.x; x[1] = v.y;
        } else if constexpr (sizeof(T) == 2 && T2 == 2) {
            const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
            x[0] = __uint_as_float(v << 16); x[1] = __uint_as_float(v & 0xffff0000u);
        } else {
            x[0] = to_float(*p);
        }
    } else {
        const T* p = row_elem_ptr<D, T, WIDE>(base, j, li);
#pragma unroll
        for (int t = 0; t < T2; ++t) x[t] = to_float(p[32 * t]);
    }
}

// Rows [row0, row0 + rows) of a [..][D] fp32 array as a raw buffer: stores through it at byte offsets at or
// beyond rows * D * 4 are dropped by the hardware, so a tile's stores need neither predicates nor 64-bit
// address arithmetic (vector instructions that an fp32 MFMA kernel pays for in matrix time).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_window(float* __restrict__ base, long long row0, int rows, int D)
{
    constexpr int kRawDword = 0x00020000;      // word 3 of a gfx9 buffer descriptor: 32-bit data format, no swizzling
    // The arguments are the same in every lane; saying so keeps the descriptor in scalar registers (otherwise each
    // store is wrapped in a loop over the distinct descriptors of the wavefront).
    const unsigned long long addr = reinterpret_cast<unsigned long long>(base + row0 * D);
    const unsigned lo = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(addr));
    const unsigned hi = __builtin_amdgcn_readfirstlane(static_cast<unsigned>(addr >> 32));
    float* uniform_base = reinterpret_cast<float*>((static_cast<unsigned long long>(hi) << 32) | lo);
    return __builtin_amdgcn_make_buffer_rsrc(uniform_base, 0, __builtin_amdgcn_readfirstlane(rows * D * 4), kRawDword);
}

// (slice, bucket) of a one-wavefront workgroup in a grid of one workgroup per bucket.  Workgroups go to the eight
// XCDs round-robin by id and start in id order.  spread_xcds: each XCD takes one contiguous eighth of all buckets,
// so the XCDs work in different slices (right when eight slices' tensors fit the Infinity Cache with room to spare:
// their reads then spread over the memory side).  Otherwise the buckets of one slice after the other, each XCD a
// contiguous eighth of the slice: one slice's tensors hot at a time.  B*H*n < 2^31, so 32-bit divisions do.
struct BucketId { uint32_t slice, l; };
__device__ __forceinline__ BucketId bucket_of_workgroup(long long n, int spread_xcds)
{
    const uint32_t n32 = static_cast<uint32_t>(n);
    BucketId b;
    if (spread_xcds) {
        const uint32_t wave = static_cast<uint32_t>(xcd_contiguous_block(blockIdx.x, gridDim.x));
        b.slice = wave / n32;
        b.l = wave - b.slice * n32;
    } else {
        b.slice = blockIdx.x / n32;
        b.l = static_cast<uint32_t>(xcd_contiguous_block(blockIdx.x - b.slice * n32, n32));
    }
    return b;
}

// What the first contraction accumulates besides the D x D tile.
enum : int {
    kExtraSumA = 0,        // column sums of the A operands        (z_l of the forward pass)
    kExtraSumB = 1,        // column sums of the B operands
    kExtraScaledSumB = 2,  // sum over contributors of escale[row] * (B operands)
    kExtraNone = 3,
};

// (row, weight[, scale]) of up to 128 consecutive entries of a column list, one entry per lane in two register
// sets: entries block + lane and block + 64 + lane, clamped to the last entry, with weight 0 past the end.
struct ListBlock {
    int32_t j_a, j_b;
    float g_a, g_b, e_a, e_b;
};

template <bool SCALED>
__device__ __forceinline__ ListBlock load_list_block(const int32_t* __restrict__ csc_row, const float* __restrict__ vals,
                                                     const float* __restrict__ escale, int32_t block, int32_t end)
{
    ListBlock b = {0, 0, 0.0f, 0.0f, 0.0f, 0.0f};
    if (block >= end) return b;       // wave-uniform
    const int lane = lane_id();
    const int32_t ea = min(block + lane, end - 1), eb = min(block + kWave + lane, end - 1);
    b.j_a = csc_row[ea]; b.j_b = csc_row[eb];
    const float va = vals[ea], vb = vals[eb];
    b.g_a = block + lane < end ? va : 0.0f;
    b.g_b = block + kWave + lane < end ? vb : 0.0f;
    if constexpr (SCALED) { b.e_a = escale[b.j_a]; b.e_b = escale[b.j_b]; }
    return b;
}

// First contraction of a bucket, shared by the bucket-forming, the bucket-fused and the backward kernels:
//     acc[a][c] (32x32 tiles) += A^T B over the column list [beg, end) of bucket l,   extra[...] += see above,
// where one of the two operands of a contributor is weight * phi(row) (A if WEIGHT_ON_A, else B) and the other
// its row as stored.  The two half-waves carry the two contributors of a pair (the k index of
// v_mfma_f32_32x32x2_f32); see load_operand_elems for which element a lane holds.
//
// On gfx950 an fp32 MFMA occupies the vector ALU: vector instructions do not issue in its shadow, so each one
// between the MFMAs is paid in matrix time.  The loop is therefore written for few vector instructions per pair:
//   - the column list is walked in blocks of 128 entries (64 contributor pairs; most lists fit in one) whose
//     (row, weight) are fetched up front (load_list_block; the first block is handed in by the caller, who can
//     fetch it while the previous bucket is still being worked on), one entry per lane in two register pairs;
//   - a lane takes its contributor's entry from there with ds_bpermute (entry 2p for the lower half-wave, 2p + 1
//     for the upper): an LDS-crossbar instruction, issued before the pair's MFMAs and complete when they are;
//   - the row address is one 32-bit multiply-add on a scalar base (row_elem_ptr), shared by both operands' loads
//     when they have the same element size;
//   - a pair's rows are fetched RING pairs ahead into a ring of RING register slots, the slot that the current
//     pair has just vacated; row loads are unconditional (pairs past the end re-read the last entry with weight
//     0), since a load skipped on one control path would force a full wait where the paths join.
template <int D, typename TA, typename TB, bool INTERLEAVED, bool WEIGHT_ON_A, int EXTRA, int FM, bool WIDE>
__device__ __forceinline__ void bucket_first_contraction(const TA* __restrict__ Ab, const TB* __restrict__ Bb,
                                                         const int32_t* __restrict__ csc_row, const float* __restrict__ vals,
                                                         const float* __restrict__ escale,
                                                         int32_t beg_in, int32_t end_in, const ListBlock& first,
                                                         floatx16 (&acc)[D / 32][D / 32], float (&zacc)[D / 32])
{
    constexpr int T2 = D / 32;
    constexpr int RING = 4;
    constexpr bool SCALED = EXTRA == kExtraScaledSumB;
    const int32_t beg = beg_in, end = end_in;
    const int lane = lane_id();
    const int li = lane & 31;
    const int pick = (lane >> 5) << 2;      // ds_bpermute byte address of lane 0 (lower half-wave) or lane 1 (upper)
#pragma unroll
    for (int a = 0; a < T2; ++a) {
        zacc[a] = 0.0f;
#pragma unroll
        for (int c = 0; c < T2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.0f;
    }
    if (beg >= end) return;

    // this lane's contributor of the pair held in lanes (s, s + 1) of (jv, gv, ev), and its two operand rows
    auto row_load = [&](int32_t jv, float gv, float ev, int first_lane, int s, float (&aa)[T2], float (&bb)[T2], float& gg, float& ee) {
        const int addr = first_lane + 4 * s;      // s is a compile-time constant at every call: one add of a literal
        const uint32_t j = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr, jv));
        gg = __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(gv)));
        if constexpr (SCALED) ee = __int_as_float(__builtin_amdgcn_ds_bpermute(addr, __float_as_int(ev)));
        load_operand_elems<D, TA, INTERLEAVED, WIDE>(Ab, j, li, aa);
        load_operand_elems<D, TB, INTERLEAVED, WIDE>(Bb, j, li, bb);
    };

    auto run_block = [&](const ListBlock& lb, int32_t block) {
        const int32_t j_a = lb.j_a, j_b = lb.j_b;
        const float g_a = lb.g_a, g_b = lb.g_b, e_a = lb.e_a, e_b = lb.e_b;
        const int pairs = min((end - block + 1) >> 1, kWave);      // pairs of this block

        float ab[RING][T2], bb[RING][T2], gb[RING], eb_[RING];
#pragma unroll
        for (int u = 0; u < RING; ++u) {
            row_load(j_a, g_a, e_a, pick, 2 * u, ab[u], bb[u], gb[u], eb_[u]);
            if ((u & 3) == 3) __builtin_amdgcn_sched_barrier(0);      // bounds the entries in flight between crossbar and loads
        }
#pragma nounroll
        for (int q0 = 0; q0 < pairs; q0 += RING) {      // kept a loop: unrolled over its at most 64 / RING rounds, the steps' waits degrade
            // this round fetches pairs q0 + RING .. q0 + 2 RING - 1 of the block: lanes of j_a for pairs
            // below 32, of j_b above (past pair 63 the fetch is redundant and re-reads j_b's tail)
            const int ahead = q0 + RING;
            const bool second = ahead >= 32;
            const int32_t j_sel = second ? j_b : j_a;
            const float g_sel = second ? g_b : g_a;
            const float e_sel = second ? e_b : e_a;
            // ds_bpermute address of the round's first pair; opaque to the optimiser, which would otherwise keep
            // sixteen loop-invariant addresses in registers and lose a wavefront of occupancy
            int lane0 = pick + 4 * ((2 * ahead) & (kWave - 1));
            asm volatile("" : "+v"(lane0));
#pragma unroll
            for (int u = 0; u < RING; ++u) {
                if (q0 + u < pairs) {
                    float a_op[T2], b_op[T2];
#pragma unroll
                    for (int t = 0; t < T2; ++t) {
                        a_op[t] = WEIGHT_ON_A ? gb[u] * feature_ct<FM>(ab[u][t]) : ab[u][t];
                        b_op[t] = WEIGHT_ON_A ? bb[u][t] : gb[u] * feature_ct<FM>(bb[u][t]);
                        if constexpr (EXTRA == kExtraSumA) zacc[t] += a_op[t];
                        if constexpr (EXTRA == kExtraSumB) zacc[t] += b_op[t];
                        if constexpr (SCALED) zacc[t] = fmaf(eb_[u], b_op[t], zacc[t]);
                    }
#pragma unroll
                    for (int a = 0; a < T2; ++a)
#pragma unroll
                        for (int c = 0; c < T2; ++c)
                            acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_op[a], b_op[c], acc[a][c], 0, 0, 0);
                }
                row_load(j_sel, g_sel, e_sel, lane0, 2 * u, ab[u], bb[u], gb[u], eb_[u]);     // into the slot just vacated
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // The first block stands apart from the loop over the others: at a loop head the compiler's load-counter
    // bookkeeping has to cover the back edge, where a list block has just been requested, and would wait for every
    // outstanding load and store there, the caller's prefetches for its second stage and (in a kernel that walks
    // over buckets) the previous bucket's stores included.
    run_block(first, beg);
    for (int32_t block = beg + 2 * kWave; block < end; block += 2 * kWave)
        run_block(load_list_block<SCALED>(csc_row, vals, escale, block, end), block);
}

// Number of one-wavefront workgroups that are resident at once for `kernel` on the current device (compute
// units x workgroups per unit at the kernel's register use), capped by the number of work items: the grid of
// the kernels that loop over their work items with a stride of the grid size.
unsigned resident_wave_grid(const void* kernel, long long items);

inline unsigned blocks_for(long long items, int per_block) { return static_cast<unsigned>((items + per_block - 1) / per_block); }

// Launch shape of the d = 64 S_l kernels (for_each_long_bucket): true when the mean list length says that few lists are
// longer than kGramMaxList.  Either shape is correct for any input and gives the same bits.
inline bool few_long_lists(int64_t n, int64_t nnz) { return nnz < 48 * n; }

// True when a [n][d] slice may span 4 GiB or more (or the test hook forces it): the bucket kernels then use
// 64-bit row offsets (row_elem_ptr).
bool wide_offsets(int64_t n, int32_t d);

// Dispatch on (d, dtype) to the compiled instances.
#define GRF_DISPATCH(d, dtype, CALL)                                                     \
    do {                                                                                 \
        if ((d) == 64 && (dtype) == GRF_DTYPE_F32) { constexpr int D_ = 64; using T_ = float; CALL; }  \
        else if ((d) == 64) { constexpr int D_ = 64; using T_ = bf16_t; CALL; }          \
        else if ((dtype) == GRF_DTYPE_F32) { constexpr int D_ = 32; using T_ = float; CALL; }          \
        else { constexpr int D_ = 32; using T_ = bf16_t; CALL; }                         \
    } while (0)

}  // namespace grf
