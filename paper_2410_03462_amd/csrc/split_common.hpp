// Shared by the d = 64 bucket kernels that run on the bf16 matrix cores: fp32 numbers as sums of bf16 pieces, the
// products of such operands as bf16 MFMAs, row loads in the kernels' element order, the walk over a column list and
// the store of an output tile.
//
// Index convention of these kernels: MFMA row/column x of tile t stands for element 2x + t of a row (a lane's two
// tiles are the two halves of one load).  Lane L = 32 g + f; in every operand the lanes of group g carry depth slots
// (g, 0..7) of v_mfma_f32_32x32x16_bf16, two bf16 per register.
#pragma once

#include "attention_common.hpp"

namespace grf {

// The bucket passes: the forward pass and the three passes of the backward pass (see backward_split.hpp).
enum : int { kQuerySide = 0, kKeySide = 1, kValueSide = 2, kForwardSide = 3 };

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

// Two fp32 numbers as one register of two bf16 (round to nearest even), x in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float x, float y)
{
    const floatx2 v = {x, y};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float low_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float high_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// x minus the low (minus_low_bf16) or high (minus_high_bf16) bf16 of w, exactly: one v_dot2c_f32_bf16 each, x + w . (-1, 0)
// or x + w . (0, -1), instead of a shift or mask and a subtraction.  (Every intermediate value is an fp32 number, so
// the result does not depend on how the instruction orders its three terms.)
// The selector pairs are handed over in registers: written as literals, the compiler encodes (-1, 0) as the inline
// constant -1.0, which the instruction does not read as a bf16 pair.
__device__ __forceinline__ uint32_t opaque_word(uint32_t w)
{
    asm("" : "+s"(w));      // not volatile: identical uses are merged into one scalar register
    return w;
}
__device__ __forceinline__ float minus_low_bf16(float x, uint32_t w)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, opaque_word(0x0000bf80u)), x, false);
}
__device__ __forceinline__ float minus_high_bf16(float x, uint32_t w)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, opaque_word(0xbf800000u)), x, false);
}

// (x, y) as hi + lo, two bf16 numbers each.
__device__ __forceinline__ void split_bf16(float x, float y, uint32_t& hi, uint32_t& lo)
{
    hi = pack_bf16(x, y);
    lo = pack_bf16(minus_low_bf16(x, hi), minus_high_bf16(y, hi));
}

__device__ __forceinline__ uint32_t low_halves(uint32_t x, uint32_t y) { return (x & 0xffffu) | (y << 16); }
__device__ __forceinline__ uint32_t high_halves(uint32_t x, uint32_t y) { return (x >> 16) | (y & 0xffff0000u); }

// max(., floor) of both 16-bit halves as signed integers: with floor = 0 this is ReLU of two bf16 numbers
// (sign-magnitude floats order like integers where it matters, see relu()), with floor = -32768 the identity.
__device__ __forceinline__ uint32_t max_i16x2(uint32_t x, uint32_t floor)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(shortx2, x), __builtin_bit_cast(shortx2, floor)));
}

__device__ __forceinline__ bf16x8 as_operand(const uint32_t (&w)[4])
{
    const uintx4 v = {w[0], w[1], w[2], w[3]};
    return __builtin_bit_cast(bf16x8, v);
}

// Walks the column list [beg, end) in steps of 16 members, out of blocks of 128 entries held one per lane in two
// register sets (load_list_block).  request(rows, weights, scales, first, set) issues the loads of the step whose
// members are entries first .. first + 15 (mod 64) of the registers handed over, into `set`; contract(set, weights,
// scales, first) does the step's arithmetic.  Two sets take turns, so that the next step's loads are in flight
// under this step's arithmetic, with scheduling barriers between request and arithmetic (the compiler would
// otherwise reorder them).  The steps come in pairs: the second one is contracted also when it lies past the end of
// the list (its members then have weight 0), since a skipped step's loads would be moved into the branch, next to
// their use; past a block's last step the request is redundant and re-reads entries of the block.  (Lists of at most
// kGramMaxList entries never come here: gram_bucket_kernel takes them.)
template <typename Members, bool SCALED, typename Request, typename Contract>
__device__ __forceinline__ void walk_column_list(const int32_t* __restrict__ csc_row, const float* __restrict__ vals,
                                                 const float* __restrict__ escale, int32_t beg, int32_t end,
                                                 Request&& request, Contract&& contract)
{
    for (int32_t block = beg; block < end; block += 2 * kWave) {
        ListBlock lb = load_list_block<SCALED>(csc_row, vals, escale, block, end);
        // all of the block's loads are taken here, where the first are needed anyway: requested later (the compiler
        // sinks the second set to its first use), they would return behind the rows' loads
        asm volatile("" : "+v"(lb.j_a), "+v"(lb.j_b), "+v"(lb.g_a), "+v"(lb.g_b), "+v"(lb.e_a), "+v"(lb.e_b));
        const int steps = min((end - block + 15) >> 4, 8);
        Members even, odd;
        __builtin_amdgcn_sched_barrier(0);
        request(lb.j_a, lb.g_a, lb.e_a, 0, even);
#pragma nounroll
        for (int s = 0; s < steps; s += 2) {
            __builtin_amdgcn_sched_barrier(0);
            request(s + 1 >= 4 ? lb.j_b : lb.j_a, s + 1 >= 4 ? lb.g_b : lb.g_a, s + 1 >= 4 ? lb.e_b : lb.e_a, 16 * (s + 1), odd);
            __builtin_amdgcn_sched_barrier(0);
            contract(even, s >= 4 ? lb.g_b : lb.g_a, s >= 4 ? lb.e_b : lb.e_a, 16 * s);
            __builtin_amdgcn_sched_barrier(0);
            request(s + 2 >= 4 ? lb.j_b : lb.j_a, s + 2 >= 4 ? lb.g_b : lb.g_a, s + 2 >= 4 ? lb.e_b : lb.e_a, 16 * (s + 2), even);
            __builtin_amdgcn_sched_barrier(0);
            contract(odd, s + 1 >= 4 ? lb.g_b : lb.g_a, s + 1 >= 4 ? lb.e_b : lb.e_a, 16 * (s + 1));
        }
    }
}

// A 32 x 64 output tile of the second contraction: register r of p0 / p1 in lane (g, f) is consumer row
// 8 (r / 4) + 4 g + r % 4, column 2 f / 2 f + 1.  One 8-byte store per register pair through a window over the
// tile's `rows` valid rows of the [..][64] fp32 array, which drops the rows past the end of the list; the rows'
// constant offsets go into the instructions' offset fields (lane_off is made opaque so that they are not hoisted
// into sixteen registers).
__device__ __forceinline__ void store_consumer_tile(float* __restrict__ partial, long long row0, int rows, int g, int f,
                                                    const floatx16& p0, const floatx16& p1)
{
    constexpr int D = 64;
    const __amdgpu_buffer_rsrc_t window = row_window(partial, row0, rows, D);
    int lane_off = (4 * g * D + 2 * f) * 4;
    asm volatile("" : "+v"(lane_off));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uintx2 v = {__float_as_uint(p0[r]), __float_as_uint(p1[r])};
        __builtin_amdgcn_raw_buffer_store_b64(v, window, lane_off + (8 * (r / 4) + (r % 4)) * D * 4, 0, 0);
    }
}

// Which bucket(s) a one-wavefront workgroup of the d = 64 S_l kernels takes.  Unless LISTED, the grid has one workgroup
// per (slice, bucket) and short lists return at once: right when most lists are long.  LISTED: a resident grid strides
// through the (slice, long bucket) pairs of the plan's list of long buckets: right when few lists are long, where a
// grid of mostly empty workgroups costs more than the work (0.2 us each).  The arithmetic per bucket is the same.
template <bool LISTED, typename Body>
__device__ __forceinline__ void for_each_long_bucket(long long n, long long n_waves, int spread_xcds,
                                                     const int32_t* __restrict__ long_list, const int32_t* __restrict__ plan_counts,
                                                     Body&& body)
{
    if constexpr (LISTED) {
        const uint32_t n_long = static_cast<uint32_t>(plan_counts[kPlanLong]);
        if (n_long == 0) return;
        const uint32_t total = static_cast<uint32_t>(n_waves / n) * n_long;      // <= B*H*n < 2^31
        for (uint32_t t = blockIdx.x; t < total; t += gridDim.x) {
            const uint32_t slice = t / n_long;
            body(slice, static_cast<uint32_t>(long_list[t - slice * n_long]));
        }
    } else {
        if (blockIdx.x >= n_waves) return;
        const BucketId bucket = bucket_of_workgroup(n, spread_xcds);
        body(bucket.slice, bucket.l);
    }
}

// (x, y) as h + m + l, two bf16 numbers each.
__device__ __forceinline__ void split3_bf16(float x, float y, uint32_t& h, uint32_t& m, uint32_t& l)
{
    h = pack_bf16(x, y);
    const float rx = minus_low_bf16(x, h), ry = minus_high_bf16(y, h);
    m = pack_bf16(rx, ry);
    l = pack_bf16(minus_low_bf16(rx, m), minus_high_bf16(ry, m));
}

// acc += a b for operands given as three pieces each: the six products that matter, small ones first.
__device__ __forceinline__ void mfma_split3(const uint32_t (&a)[3][4], const uint32_t (&b)[3][4], floatx16& acc)
{
    const bf16x8 ah = as_operand(a[0]), am = as_operand(a[1]), al = as_operand(a[2]);
    const bf16x8 bh = as_operand(b[0]), bm = as_operand(b[1]), bl = as_operand(b[2]);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
}

// The same for operands in NP pieces (3, or 2 where a relative error of 2^-16 per operand is within the bar: bf16 inputs).
template <int NP>
__device__ __forceinline__ void split_pieces(float x, float y, uint32_t (&dst)[NP][4], int p)
{
    if constexpr (NP == 3) split3_bf16(x, y, dst[0][p], dst[1][p], dst[2][p]);
    else split_bf16(x, y, dst[0][p], dst[1][p]);
}
template <int NP>
__device__ __forceinline__ void mfma_pieces(const uint32_t (&a)[NP][4], const uint32_t (&b)[NP][4], floatx16& acc)
{
    if constexpr (NP == 3) {
        mfma_split3(a, b, acc);
    } else {
        const bf16x8 ah = as_operand(a[0]), al = as_operand(a[1]), bh = as_operand(b[0]), bl = as_operand(b[1]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc, 0, 0, 0);
    }
}

// Elements 2f, 2f + 1 of a row as loaded (one 8-byte or one 4-byte load), widened to fp32 only where they are used.
template <typename T> struct RawPair { typedef float2 type; };
template <> struct RawPair<bf16_t> { typedef uint32_t type; };

template <typename T, bool WIDE>
__device__ __forceinline__ typename RawPair<T>::type load_pair(const T* __restrict__ base, uint32_t row, int f)
{
    return *reinterpret_cast<const typename RawPair<T>::type*>(row_elem_ptr<64, T, WIDE>(base, row, 2 * f));
}
__device__ __forceinline__ float2 widen(float2 v) { return v; }
__device__ __forceinline__ float2 widen(uint32_t w) { return make_float2(low_bf16(w), high_bf16(w)); }

// Eight consecutive elements of a row starting at element `elem` (a multiple of 8), widened to fp32.
template <typename T, bool WIDE>
__device__ __forceinline__ void load_eight(const T* __restrict__ base, uint32_t row, int elem, float (&x)[8])
{
    if constexpr (sizeof(T) == 4) {
        const float4* p = reinterpret_cast<const float4*>(row_elem_ptr<64, T, WIDE>(base, row, elem));
        const float4 u = p[0], v = p[1];
        x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; x[4] = v.x; x[5] = v.y; x[6] = v.z; x[7] = v.w;
    } else {
        const uintx4 w = *reinterpret_cast<const uintx4*>(row_elem_ptr<64, T, WIDE>(base, row, elem));
#pragma unroll
        for (int k = 0; k < 4; ++k) { x[2 * k] = low_bf16(w[k]); x[2 * k + 1] = high_bf16(w[k]); }
    }
}

}  // namespace grf
