// Random-walk sampler and CSR assembly of the GRF matrix Phi_hat (Alg. 1 steps 1-2; Sec. 3.3).
//
// One wavefront owns one start node: its lanes run that node's walks in lock step, deposit
// (column, load, hop) triples into LDS, order them by column with a rank-by-counting pass and
// merge equal columns.  The kernel runs twice, first to count the entries of every row and,
// after an exclusive scan, to write them at their final place, so no worst-case staging buffer
// exists in HBM.  Walk decisions are integer-only (Philox words, a threshold compare and a
// multiply-high), hence trajectories and the sparsity pattern do not depend on floating point.
#include <atomic>
#include <cmath>
#include <type_traits>

#include "common.hpp"

namespace grf {

// ------------------------------------------------------------------------------------ Philox
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and xors with
// a Weyl-sequence key schedule.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // both halves of a product from one 32 x 32 -> 64 bit multiply (a quarter-rate instruction, as each of a
        // separate high and low multiply would be: the walks' arithmetic is mostly these)
        const uint64_t p0 = static_cast<uint64_t>(M0) * c0, p1 = static_cast<uint64_t>(M1) * c2;
        const uint32_t hi0 = static_cast<uint32_t>(p0 >> 32), lo0 = static_cast<uint32_t>(p0);
        const uint32_t hi1 = static_cast<uint32_t>(p1 >> 32), lo1 = static_cast<uint32_t>(p1);
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

struct GraphView {
    const int32_t* row_ptr;
    const int32_t* col;
    const float* w;
    int32_t n;
    int32_t nnz;
};

struct WalkLaw {
    uint32_t key0, key1;      // Philox key = (seed low word, seed high word)
    uint32_t threshold;       // halt iff draw < threshold ...
    int32_t always_halt;      // ... or always, when p_halt = 1 makes the threshold 2^32
    float inv_survive;        // 1 / (1 - p_halt)
};

// One hop of one walk.  `x` holds the Philox block serving hops 2b+1 (words 0,1) and 2b+2
// (words 2,3).  Returns false when the walk ends before this hop (isolated node, halting draw,
// or a malformed graph entry, which is treated as a dead end rather than followed out of bounds).
__device__ __forceinline__ bool walk_hop(const GraphView& g, const WalkLaw& law, int t,
                                         const uint32_t (&x)[4], int32_t& u, float& load)
{
    const int32_t beg = g.row_ptr[u];
    const int32_t end = g.row_ptr[u + 1];
    const int32_t deg = end - beg;
    if (deg <= 0 || beg < 0 || end > g.nnz) return false;
    const bool second = ((t - 1) & 1) != 0;
    const uint32_t draw_halt = second ? x[2] : x[0];
    const uint32_t draw_nbr = second ? x[3] : x[1];
    if (law.always_halt || draw_halt < law.threshold) return false;
    const int32_t e = beg + static_cast<int32_t>(__umulhi(draw_nbr, static_cast<uint32_t>(deg)));
    const int32_t v = g.col[e];
    if (static_cast<uint32_t>(v) >= static_cast<uint32_t>(g.n)) return false;
    // importance weight of the prefix: edge weight over transition probability (1-p)/deg
    load *= g.w[e] * (static_cast<float>(deg) * law.inv_survive);
    u = v;
    return true;
}

// ------------------------------------------------------------------------------------ trajectories
__global__ __launch_bounds__(256) void walks_kernel(GraphView g, WalkLaw law, int n_walks, int max_nodes,
                                                    int32_t* __restrict__ traj)
{
    const long long gid = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (gid >= static_cast<long long>(g.n) * n_walks) return;
    const uint32_t node = static_cast<uint32_t>(gid / n_walks);
    const uint32_t walk = static_cast<uint32_t>(gid % n_walks);
    int32_t* out = traj + gid * max_nodes;
    int32_t u = static_cast<int32_t>(node);
    float load = 1.0f;
    bool alive = true;
    uint32_t x[4] = {0, 0, 0, 0};
    out[0] = u;
    for (int t = 1; t < max_nodes; ++t) {
        if (((t - 1) & 1) == 0) philox4x32_10(node, walk, static_cast<uint32_t>((t - 1) >> 1), 0u, law.key0, law.key1, x);
        if (alive) alive = walk_hop(g, law, t, x, u, load);
        out[t] = alive ? u : -1;
    }
}

// ------------------------------------------------------------------------------------ rows of Phi_hat
// LDS layout for `cap` deposits: dcol[cap] dload[cap] (4 B each), dhop[cap] perm[cap] (2 B each) = 12 B per
// deposit, plus dent[cap] (4 B) in the gradient mode.  The deposits stay where the walks put them; the column
// order is an index permutation (perm[r] = deposit at sorted position r), which keeps the footprint small, so that
// enough wavefronts fit a compute unit to cover the hops' dependent loads and keep its vector ALUs issuing.
constexpr int kDepositBytes = 12;
// testing aid (grf_debug_force_row_kernel): 1 = wavefront kernel, 2 = workgroup kernel wherever both can serve;
// 3 = wavefront kernel ordering by (column, slot) as two words, the form it takes when they do not fit one
std::atomic<int> g_force_row_kernel{0};
constexpr int kDepositBytesGrad = 16;

// rank += (a < b), unsigned, as a compare into the carry flag and an add with carry: two vector instructions (written
// as `rank += a < b` the comparison goes through a scalar register pair and a select: four, with a wait in between).
__device__ __forceinline__ void count_below(int& rank, uint32_t a, uint32_t b)
{
    asm("v_cmp_lt_u32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, 0, %0, vcc" : "+v"(rank) : "v"(a), "v"(b) : "vcc");
}

// MODE kCount: row_ptr[node] = number of entries of the row.  kFill: entries written at row_ptr[node].
// kGrad: instead of values, the row's share of dL/df is written to df_part[node][n_f][f_len], where
// dphi ([n_f][val_stride]) holds dL/dPhi_hat per stored entry.
enum : int { kCount = 0, kFill = 1, kGrad = 2 };

// A wavefront serves 64 / W start nodes, W lanes each (W = the smallest of 8, 16, 32, 64 that covers n_walks, so
// that few lanes idle: the kernel is bound by vector-instruction issue, and a wavefront's hops and Philox blocks
// cost the same instructions however many of its lanes walk).  `sub` is the node's slot in the wavefront, `sl` the lane in it.
template <int MODE, int W, bool PACKED>
__global__ __launch_bounds__(64) void rows_kernel(GraphView g, WalkLaw law, int n_walks, int f_len, int n_f,
                                                  const float* __restrict__ f, int cap, int slot_bits,
                                                  int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_out,
                                                  float* __restrict__ val_out, long long val_stride,
                                                  const float* __restrict__ dphi, float* __restrict__ df_part)
{
    constexpr bool FILL = MODE == kFill;
    constexpr int P = kWave / W;
    constexpr int kBytes = MODE == kGrad ? kDepositBytesGrad : kDepositBytes;
    const int lane = threadIdx.x;
    const int sub = lane / W;
    const int sl = lane % W;
    // this node's share of a wave-wide ballot, and the number of its set bits below this lane
    auto share = [&](unsigned long long mask) -> unsigned long long {
        if constexpr (W == kWave) return mask;
        else return (mask >> (W * sub)) & ((1ull << W) - 1ull);
    };
    auto below = [&](unsigned long long mine) { return __popcll(mine & ((1ull << sl) - 1ull)); };

    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char* region = lds + static_cast<size_t>(sub) * cap * kBytes;
    int32_t* dcol = reinterpret_cast<int32_t*>(region);
    float* dload = reinterpret_cast<float*>(dcol + cap);
    uint16_t* dhop = reinterpret_cast<uint16_t*>(dload + cap);
    uint16_t* perm = dhop + cap;
    int32_t* dent = reinterpret_cast<int32_t*>(perm + cap);      // gradient mode only; byte offset 12 cap: 4-byte aligned

    const long long node_ll = static_cast<long long>(blockIdx.x) * P + sub;
    const bool has_node = node_ll < g.n;
    const uint32_t node = static_cast<uint32_t>(has_node ? node_ll : 0);

    // The n_walks zero-hop prefixes all deposit load 1 at the start node: one merged deposit.
    // PACKED: dcol holds (column << slot_bits | slot), one unsigned key whose order is the order (column, slot)
    auto stored = [&](int32_t column, int slot) -> int32_t {
        if constexpr (PACKED) return static_cast<int32_t>((static_cast<uint32_t>(column) << slot_bits) | static_cast<uint32_t>(slot));
        else return column;
    };
    auto column_of = [&](int32_t held) -> int32_t {
        if constexpr (PACKED) return static_cast<int32_t>(static_cast<uint32_t>(held) >> slot_bits);
        else return held;
    };
    if (sl == 0 && has_node) { dcol[0] = stored(static_cast<int32_t>(node), 0); dload[0] = static_cast<float>(n_walks); dhop[0] = 0; }
    int base = has_node ? 1 : 0;
    for (int first = 0; first < n_walks; first += W) {
        const uint32_t walk = static_cast<uint32_t>(first + sl);
        bool alive = has_node && static_cast<int>(walk) < n_walks;
        int32_t u = static_cast<int32_t>(node);
        float load = 1.0f;
        uint32_t x[4] = {0, 0, 0, 0};
        for (int t = 1; t < f_len; ++t) {
            if (((t - 1) & 1) == 0) philox4x32_10(node, walk, static_cast<uint32_t>((t - 1) >> 1), 0u, law.key0, law.key1, x);
            if (alive) alive = walk_hop(g, law, t, x, u, load);
            const unsigned long long mask = __ballot(alive);
            if (mask == 0ull) break;
            const unsigned long long mine = share(mask);
            if (alive) {
                const int pos = base + below(mine);
                dcol[pos] = stored(u, pos); dload[pos] = load; dhop[pos] = static_cast<uint16_t>(t);
            }
            base += __popcll(mine);
        }
    }
    const int D = base;   // <= 1 + n_walks * (f_len - 1) <= cap; 0 in a slot without a node
    int d_max = D;        // the largest D of the wavefront: bound of the loops that hold a ballot
#pragma unroll
    for (int off = W; off < kWave; off <<= 1) d_max = max(d_max, __shfl_xor(d_max, off, kWave));
    if constexpr (PACKED) {
        // the ranking reads sixteen keys at a time: the last group is filled up with keys above all others
        for (int j = D + sl; j < ((D + 15) & ~15); j += W) dcol[j] = -1;
    }
    __syncthreads();

    // Rank by counting: position of deposit s in the order (column, s).
    if constexpr (PACKED) {
        const uint32_t* key = reinterpret_cast<const uint32_t*>(dcol);
        for (int s = sl; s < D; s += W) {
            const uint32_t k = key[s];
            int rank = 0;
            for (int s2 = 0; s2 < D; s2 += 16) {      // the region is 16-byte aligned (cap is a multiple of 16)
                const uint4* k4 = reinterpret_cast<const uint4*>(key + s2);
                const uint4 a = k4[0], b = k4[1], c = k4[2], d = k4[3];      // four reads in flight, then 32 instructions
                count_below(rank, a.x, k); count_below(rank, a.y, k); count_below(rank, a.z, k); count_below(rank, a.w, k);
                count_below(rank, b.x, k); count_below(rank, b.y, k); count_below(rank, b.z, k); count_below(rank, b.w, k);
                count_below(rank, c.x, k); count_below(rank, c.y, k); count_below(rank, c.z, k); count_below(rank, c.w, k);
                count_below(rank, d.x, k); count_below(rank, d.y, k); count_below(rank, d.z, k); count_below(rank, d.w, k);
            }
            perm[rank] = static_cast<uint16_t>(s);
        }
    } else {
        for (int s = sl; s < D; s += W) {
            const int32_t c = dcol[s];
            int rank = 0;
            for (int s2 = 0; s2 < D; ++s2) {
                const int32_t c2 = dcol[s2];
                rank += static_cast<int>((c2 < c) | ((c2 == c) & (s2 < s)));
            }
            perm[rank] = static_cast<uint16_t>(s);
        }
    }
    __syncthreads();

    // Runs of equal columns: the run head writes the merged entry.
    const int32_t row_start = (MODE != kCount && has_node) ? row_ptr[node] : 0;
    const float n_float = static_cast<float>(n_walks);
    int heads = 0;
    for (int r0 = 0; r0 < d_max; r0 += W) {
        const int r = r0 + sl;
        const bool valid = r < D;
        const int32_t c = valid ? column_of(dcol[perm[r]]) : -1;
        const bool head = valid && (r == 0 || column_of(dcol[perm[r - 1]]) != c);
        const unsigned long long mine = share(__ballot(head));
        if (MODE == kGrad && valid) {
            // entry of Phi_hat that sorted position r belongs to: runs up to and including this lane, minus one
            dent[r] = row_start + heads + below(mine) + (head ? 1 : 0) - 1;
        }
        if (FILL && head) {
            const long long pos = static_cast<long long>(row_start) + heads + below(mine);
            col_out[pos] = c;
            for (int h = 0; h < n_f; ++h) {
                const float* fh = f + static_cast<long long>(h) * f_len;
                // a run is summed in blocks of 32 deposits, so that the rounding of a long run (thousands of walks
                // ending at one node) grows with run / 32 + 32 terms instead of with the run
                float acc = 0.0f, part = 0.0f;
                int in_part = 0;
                for (int e = r; e < D; ++e) {
                    const int s = perm[e];
                    if (column_of(dcol[s]) != c) break;
                    part = fmaf(dload[s], fh[dhop[s]], part);
                    if (++in_part == 32) { acc += part; part = 0.0f; in_part = 0; }
                }
                acc += part;
                val_out[h * val_stride + pos] = acc / n_float;
            }
        }
        heads += __popcll(mine);
    }
    if (MODE == kCount && sl == 0 && has_node) row_ptr[node] = heads;

    if (MODE == kGrad) {
        // dL/df[h][t] of this node = (1/n) sum over deposits with hop t of load * dphi[h][entry]; lane t walks
        // the deposits in sorted order, so the sum has a fixed order.  The columns are not needed any more:
        // their array holds the staged products.
        float* gval = reinterpret_cast<float*>(dcol);
        const int32_t row_end = has_node ? row_ptr[node + 1] : 0;
        for (int h = 0; h < n_f; ++h) {
            __syncthreads();
            for (int r = sl; r < D; r += W) {
                const int32_t e = dent[r];
                gval[r] = (e >= 0 && e < row_end && e < val_stride) ? dload[perm[r]] * dphi[h * val_stride + e] : 0.0f;
            }
            __syncthreads();
            if (has_node) {
                for (int t = sl; t < f_len; t += W) {
                    float acc = 0.0f;      // blocks of 64 deposits, as for the values
                    for (int r0 = 0; r0 < D; r0 += 64) {
                        const int r1 = min(D, r0 + 64);
                        float part = 0.0f;
                        for (int r = r0; r < r1; ++r) part += dhop[perm[r]] == t ? gval[r] : 0.0f;
                        acc += part;
                    }
                    df_part[(static_cast<long long>(node) * n_f + h) * f_len + t] = acc / n_float;
                }
            }
        }
    }
}

// Launches rows_kernel<MODE, W> with the sub-wavefront width that fits n_walks.
template <int MODE>
grf_status launch_rows(const GraphView& gv, const WalkLaw& law, int n_walks, int f_len, int n_f, const float* f, int cap,
                       int32_t* row_ptr, int32_t* col_out, float* val_out, long long val_stride, const float* dphi,
                       float* df_part, hipStream_t stream)
{
    constexpr int kBytes = MODE == kGrad ? kDepositBytesGrad : kDepositBytes;
    cap = (cap + 15) & ~15;      // the ranking reads sixteen keys at a time, in 16-byte reads: whole groups, aligned areas
    // (column, slot) as one 32-bit key while the node numbers leave room for the slot bits
    int slot_bits = 0;
    while ((1ll << slot_bits) < cap) ++slot_bits;
    const bool packed = (static_cast<long long>(gv.n) << slot_bits) <= (1ll << 32) && g_force_row_kernel.load(std::memory_order_relaxed) != 3;
    auto launch = [&](auto width) -> grf_status {
        constexpr int W = decltype(width)::value;
        constexpr int P = kWave / W;
        const size_t lds = static_cast<size_t>(P) * cap * kBytes;
        const unsigned blocks = static_cast<unsigned>((static_cast<long long>(gv.n) + P - 1) / P);
        auto go = [&](auto kernel) -> grf_status {
            if (lds > 64 * 1024)
                GRF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
            hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kWave), lds, stream, gv, law, n_walks, f_len, n_f, f, cap, slot_bits,
                               row_ptr, col_out, val_out, val_stride, dphi, df_part);
            GRF_LAUNCH_CHECK("rows_kernel");
            return GRF_OK;
        };
        return packed ? go(&rows_kernel<MODE, W, true>) : go(&rows_kernel<MODE, W, false>);
    };
    // several nodes per wavefront only while their deposit areas together stay within 8 KB, somewhat more than a wavefront
    // slot's share of a compute unit's 160 KB of LDS: beyond that the areas, not the slots, bound the nodes in flight, and
    // sharing a wavefront only stretches each node's ranking over fewer lanes (measured at the headline graph: 16 walks of
    // up to 15 hops 0.19 ms with two nodes per wavefront against 0.22 with one; the headline's 32 walks, 12 KB for two
    // nodes, 0.39 against 0.33 ms)
    auto fits = [&](int width) { return n_walks <= width && static_cast<size_t>(kWave / width) * cap * kBytes <= 8 * 1024; };
    if (fits(8)) return launch(std::integral_constant<int, 8>{});
    if (fits(16)) return launch(std::integral_constant<int, 16>{});
    if (fits(32)) return launch(std::integral_constant<int, 32>{});
    return launch(std::integral_constant<int, 64>{});
}

// ------------------------------------------------------------------------------------ rows with many deposits
// Rows whose deposits exceed what one wavefront can order by counting: one workgroup of kLargeBlock threads per node
// (a resident grid strides over the nodes), threads = walks.
//   1. Every walk is simulated twice from its counter-based stream: first for its number of hops, then, after a prefix
//      sum over the walks, to write its deposits at their slots, so that the deposits stand in (walk, hop) order.
//      Columns go to LDS with the slot number as a 16-bit tag; loads and hops go to a staging area of the workgroup in
//      the caller's workspace (they are only needed again once, by slot).
//   2. (column, slot) pairs are ordered by a bitonic sorting network in LDS (all comparators ascending, so that the
//      positions past the last deposit behave as +infinity and are skipped: no padding to a power of two).
//   3. Every thread owns a run of consecutive sorted positions: heads of equal-column runs are counted, a prefix sum
//      gives each run its entry number, and the runs' sums Sum load * f[hop] are formed per thread in sorted order and
//      joined across threads by a segmented prefix sum: a fixed order, bitwise reproducible.
// LDS: 6 bytes per possible deposit, so 16384 deposits take 96 KB.
constexpr int kLargeBlock = 1024;
constexpr int kLargeWaves = kLargeBlock / kWave;
constexpr int kLargeMaxGrid = 512;         // workgroups (and staging areas) at most
constexpr int kLargeMaxDeposits = 16384;   // 16-bit slot tags; 96 KB of LDS

// Exclusive prefix sum of one int per thread over the workgroup; *total = sum of all.  `scratch` holds kLargeWaves ints.
__device__ __forceinline__ int block_exclusive_scan(int v, int* scratch, int* total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    __syncthreads();      // scratch may still be read from a previous call
    if (lane == kWave - 1) scratch[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kLargeWaves; ++w) {
        const int t = scratch[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

// Segmented exclusive prefix sum over the workgroup's threads, in thread order: each thread contributes (value, flag);
// a set flag starts a new segment at that thread.  Returns the sum of the values of the threads before this one back to
// and including the nearest thread with a set flag (or from thread 0).
__device__ __forceinline__ float block_segmented_exclusive_sum(float v, bool flag, float* scratch_v, int* scratch_f)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    // inclusive segmented scan inside the wavefront
    float sv = v;
    int sf = flag ? 1 : 0;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const float uv = __shfl_up(sv, off, kWave);
        const int uf = __shfl_up(sf, off, kWave);
        if (lane >= off) {
            if (!sf) sv += uv;
            sf |= uf;
        }
    }
    __syncthreads();
    if (lane == kWave - 1) { scratch_v[wave] = sv; scratch_f[wave] = sf; }
    __syncthreads();
    // carry into this wavefront: the wavefronts before it, back to the nearest one that holds a flag
    float carry = 0.0f;
    for (int w = 0; w < wave; ++w) {
        if (scratch_f[w]) carry = scratch_v[w]; else carry += scratch_v[w];
    }
    // exclusive value of this thread: the inclusive value of the previous lane, joined with the carry
    float pv = __shfl_up(sv, 1, kWave);
    int pf = __shfl_up(sf, 1, kWave);
    if (lane == 0) { pv = 0.0f; pf = 0; }
    return pf ? pv : carry + pv;
}

template <int MODE>
__global__ __launch_bounds__(kLargeBlock) void rows_large_kernel(GraphView g, WalkLaw law, int n_walks, int f_len, int n_f,
                                                                 const float* __restrict__ f, int cap,
                                                                 int32_t* __restrict__ row_ptr, int32_t* __restrict__ col_out,
                                                                 float* __restrict__ val_out, long long val_stride,
                                                                 const float* __restrict__ dphi, float* __restrict__ df_part,
                                                                 float* __restrict__ stage_load, uint16_t* __restrict__ stage_hop)
{
    extern __shared__ __align__(16) unsigned char lds[];
    uint32_t* dcol = reinterpret_cast<uint32_t*>(lds);               // [cap] column of the deposit at a sorted position
    uint16_t* dslot = reinterpret_cast<uint16_t*>(dcol + cap);       // [cap] its slot in (walk, hop) order
    __shared__ int scan_i[kLargeWaves];
    __shared__ float scan_v[kLargeWaves];
    __shared__ int scan_f[kLargeWaves];
    const int tid = threadIdx.x;
    float* my_load = stage_load + static_cast<size_t>(blockIdx.x) * cap;
    uint16_t* my_hop = stage_hop + static_cast<size_t>(blockIdx.x) * cap;
    const float n_float = static_cast<float>(n_walks);

    // hops of walk `walk` out of `node` (deposit == nullptr), or its deposits written from slot `at` on
    auto run_walk = [&](uint32_t node, uint32_t walk, bool write, int at) -> int {
        int32_t u = static_cast<int32_t>(node);
        float load = 1.0f;
        uint32_t x[4] = {0, 0, 0, 0};
        int hops = 0;
        for (int t = 1; t < f_len; ++t) {
            if (((t - 1) & 1) == 0) philox4x32_10(node, walk, static_cast<uint32_t>((t - 1) >> 1), 0u, law.key0, law.key1, x);
            if (!walk_hop(g, law, t, x, u, load)) break;
            if (write) {
                const int slot = at + hops;
                dcol[slot] = static_cast<uint32_t>(u);
                dslot[slot] = static_cast<uint16_t>(slot);
                my_load[slot] = load;
                my_hop[slot] = static_cast<uint16_t>(t);
            }
            ++hops;
        }
        return hops;
    };

    for (long long node_ll = blockIdx.x; node_ll < g.n; node_ll += gridDim.x) {
        const uint32_t node = static_cast<uint32_t>(node_ll);
        __syncthreads();      // the previous node's arrays are no longer read
        // ---- 1. deposits in (walk, hop) order; the n_walks zero-hop prefixes are one deposit of load n_walks
        if (tid == 0) { dcol[0] = node; dslot[0] = 0; my_load[0] = n_float; my_hop[0] = 0; }
        int base = 1;
        for (int first = 0; first < n_walks; first += kLargeBlock) {
            const uint32_t walk = static_cast<uint32_t>(first + tid);
            const bool active = static_cast<int>(walk) < n_walks;
            const int hops = active ? run_walk(node, walk, false, 0) : 0;
            int total = 0;
            const int off = block_exclusive_scan(hops, scan_i, &total);
            if (active && hops > 0) run_walk(node, walk, true, base + off);
            base += total;
        }
        const int D = base;      // <= cap
        __syncthreads();

        // ---- 2. sort (column, slot) ascending
        int d_pad = 1;
        while (d_pad < D) d_pad <<= 1;
        auto compare_exchange = [&](int i, int j) {
            const uint32_t ci = dcol[i], cj = dcol[j];
            const uint16_t si = dslot[i], sj = dslot[j];
            if (ci > cj || (ci == cj && si > sj)) { dcol[i] = cj; dcol[j] = ci; dslot[i] = sj; dslot[j] = si; }
        };
        for (int k = 2; k <= d_pad; k <<= 1) {
            const int half = k >> 1;
            for (int p = tid; p < (d_pad >> 1); p += kLargeBlock) {      // first step of a merge: i against its mirror image
                const int blk = p / half, o = p - blk * half;
                const int i = blk * k + o, j = blk * k + k - 1 - o;
                if (j < D) compare_exchange(i, j);
            }
            __syncthreads();
            for (int j2 = half >> 1; j2 > 0; j2 >>= 1) {
                for (int p = tid; p < (d_pad >> 1); p += kLargeBlock) {
                    const int i = ((p / j2) * (j2 << 1)) + (p % j2);
                    if (i + j2 < D) compare_exchange(i, i + j2);
                }
                __syncthreads();
            }
        }

        // ---- 3. runs of equal columns; thread `tid` owns sorted positions [lo, hi)
        const int per = (D + kLargeBlock - 1) / kLargeBlock;
        const int lo = min(tid * per, D), hi = min(lo + per, D);
        auto is_head = [&](int r) { return r == 0 || dcol[r - 1] != dcol[r]; };
        int heads_mine = 0;
        for (int r = lo; r < hi; ++r) heads_mine += is_head(r) ? 1 : 0;
        int heads_total = 0;
        const int heads_before = block_exclusive_scan(heads_mine, scan_i, &heads_total);
        if (MODE == kCount) {
            if (tid == 0) row_ptr[node] = heads_total;
            continue;
        }
        const int32_t row_start = row_ptr[node];

        if (MODE == kFill) {
            const int t_last = (D - 1) / per;      // the thread that owns the last position
            for (int h = 0; h < n_f; ++h) {
                const float* fh = f + static_cast<long long>(h) * f_len;
                // sums of this thread's positions: `pre` up to its first head, then one sum per run that starts here
                float acc = 0.0f, pre = 0.0f;
                int k = 0;      // heads met so far
                for (int r = lo; r < hi; ++r) {
                    const int slot = dslot[r];
                    const float v = my_load[slot] * fh[my_hop[slot]];
                    if (is_head(r)) {
                        if (k == 0) pre = acc;
                        else {      // the run that started at this thread's head k - 1 ends before r
                            const long long pos = static_cast<long long>(row_start) + heads_before + k - 1;
                            if (h == 0) col_out[pos] = static_cast<int32_t>(dcol[r - 1]);
                            val_out[h * val_stride + pos] = acc / n_float;
                        }
                        acc = v;
                        ++k;
                    } else {
                        acc += v;
                    }
                }
                if (k == 0) pre = acc;
                // what flows into this thread from the threads before it: their sums since the nearest head
                const float carry = block_segmented_exclusive_sum(k > 0 ? acc : pre, k > 0, scan_v, scan_f);
                if (lo < hi) {
                    if (k > 0 && lo > 0) {      // the run that was open at lo ends before this thread's first head
                        const long long pos = static_cast<long long>(row_start) + heads_before - 1;
                        if (h == 0) col_out[pos] = static_cast<int32_t>(dcol[lo - 1]);
                        val_out[h * val_stride + pos] = (carry + pre) / n_float;
                    }
                    if (tid == t_last) {        // the last run of the row ends at D
                        const long long pos = static_cast<long long>(row_start) + heads_total - 1;
                        if (h == 0) col_out[pos] = static_cast<int32_t>(dcol[D - 1]);
                        val_out[h * val_stride + pos] = (k > 0 ? acc : carry + pre) / n_float;
                    }
                }
            }
        }

        if (MODE == kGrad) {
            // entry of Phi_hat of every deposit, by slot: overwrites the columns once everybody has its heads
            uint32_t ent_mine[kLargeMaxDeposits / kLargeBlock];
            {
                int k = 0;
                for (int r = lo, q = 0; r < hi; ++r, ++q) {
                    k += is_head(r) ? 1 : 0;
                    ent_mine[q] = static_cast<uint32_t>(row_start + heads_before + k - 1);
                }
            }
            __syncthreads();
            uint32_t* ent = dcol;
            for (int r = lo, q = 0; r < hi; ++r, ++q) ent[dslot[r]] = ent_mine[q];
            __syncthreads();
            // first slot of every walk (n_walks + 1 offsets, 16 bits each, where the slot tags were)
            uint16_t* first_slot = dslot;
            int base2 = 1;
            for (int first = 0; first < n_walks; first += kLargeBlock) {
                const uint32_t walk = static_cast<uint32_t>(first + tid);
                const bool active = static_cast<int>(walk) < n_walks;
                const int hops = active ? run_walk(node, walk, false, 0) : 0;
                int total = 0;
                const int off = block_exclusive_scan(hops, scan_i, &total);
                if (active) first_slot[walk] = static_cast<uint16_t>(base2 + off);
                base2 += total;
            }
            if (tid == 0) first_slot[n_walks] = static_cast<uint16_t>(base2);
            __syncthreads();
            const int32_t row_end = row_ptr[node + 1];
            const int lane = tid & (kWave - 1), wave = tid >> 6;
            for (int h = 0; h < n_f; ++h) {
                // one wavefront per hop count t: lanes stride over the walks with at least t hops, then a fixed tree
                for (int t = wave; t < f_len; t += kLargeWaves) {
                    float acc = 0.0f;
                    if (t == 0) {
                        const uint32_t e = ent[0];
                        if (lane == 0 && e < static_cast<uint32_t>(row_end) && static_cast<long long>(e) < val_stride) acc = my_load[0] * dphi[h * val_stride + e];
                    } else {
                        for (int w = lane; w < n_walks; w += kWave) {
                            const int s0 = first_slot[w], s1 = first_slot[w + 1];
                            if (s1 - s0 >= t) {
                                const int slot = s0 + t - 1;
                                const uint32_t e = ent[slot];
                                if (e < static_cast<uint32_t>(row_end) && static_cast<long long>(e) < val_stride) acc += my_load[slot] * dphi[h * val_stride + e];
                            }
                        }
                    }
                    acc = wave_sum(acc);
                    if (lane == 0) df_part[(static_cast<long long>(node) * n_f + h) * f_len + t] = acc / n_float;
                }
            }
        }
    }
}

// Which kernel assembles the rows.  Up to kLargeThreshold possible deposits the wavefront kernel always serves (and the
// workspace holds no staging areas); beyond kWaveMaxDeposits (its LDS area: 12, in the gradient mode 16 bytes per
// possible deposit) only the workgroup kernel can.  In between the cheaper one by a cost model, in microseconds per
// pass, fitted to timings of both kernels on graphs of 1024, 8192 and 32768 nodes, bounds of 769 .. 8191 deposits, with
// and without halting (it is within 25 % of them):
//   wavefront kernel   rounds of (compute units x resident wavefronts) nodes; a round costs the node's hops (the lanes'
//                      scattered loads: 0.103 per hop) plus the ranking by counting of its D deposits: 0.000112 D^2 when
//                      a SIMD holds one wavefront (the LDS reads' latency shows), 0.000013 D^2 per resident wavefront
//                      of the compute unit when it holds several (two instructions per comparison, no waits);
//   workgroup kernel   rounds of kLargeMaxGrid nodes; a round costs the two simulations of the walks (2.0 per step of the
//                      longest walk, 1.5 per hop of the average one), the barriers of the sorting network (0.4 per
//                      stage, a stage repeated for every 2048 positions) and 10 of fixed work.
// D, the hops and the longest walk are expectations under the halting law, so sparse rows of a large bound (many walks
// that halt early) stay with the wavefront kernel where it is faster (headline graph, 64 walks of up to 15 hops,
// p_halt = 0.2, bound 961, about 250 deposits: 0.8 against 7.6 ms per call) and rows filled to a large bound go to the
// workgroup kernel (32 x 32 grid, no halting, 2049 deposits: 0.66 against 1.45 ms; 8191: 1.9 against 68 ms).
constexpr int kLargeThreshold = 768;
constexpr int kWaveMaxDeposits = 8192;
inline bool large_rows_possible(long long cap) { return cap > kLargeThreshold; }
inline bool large_rows(long long n, long long cap, int n_walks, int f_len, double p_halt, int bytes_per_deposit)
{
    if (cap <= kLargeThreshold) return false;
    if (cap > kWaveMaxDeposits) return true;
    const int forced = g_force_row_kernel.load(std::memory_order_relaxed);
    if (forced == 1 || forced == 3) return false;
    if (forced == 2) return true;
    const double longest = f_len - 1;
    const double q = 1.0 - p_halt;
    double mean_hops = longest, steps = longest;
    if (p_halt > 0.0) {
        mean_hops = q > 0.0 ? q * (1.0 - std::pow(q, longest)) / p_halt : 0.0;
        const double expected_max = q > 0.0 ? std::log(static_cast<double>(n_walks < 2 ? 2 : n_walks)) / -std::log(q) + 1.0 : 1.0;
        steps = expected_max < longest ? expected_max : longest;
    }
    const double hops = n_walks * mean_hops, deposits = 1.0 + hops;

    double resident = std::floor(160.0 * 1024.0 / (static_cast<double>((cap + 15) & ~15ll) * bytes_per_deposit));
    resident = resident < 1.0 ? 1.0 : (resident > 32.0 ? 32.0 : resident);
    const double per_unit = std::ceil(static_cast<double>(n) / 256.0);      // nodes of a compute unit: fewer than fit, on a small graph
    const double sharing = resident < per_unit ? resident : per_unit;
    const double rank_us = 0.000013 * sharing > 0.000112 ? 0.000013 * sharing : 0.000112;
    const double wave_us = std::ceil(static_cast<double>(n) / (256.0 * resident)) * (0.103 * hops + rank_us * deposits * deposits);

    double positions = 64.0, log_positions = 6.0;      // the network's size: the power of two that covers the deposits
    while (positions < deposits) { positions *= 2.0; log_positions += 1.0; }
    const double stages = 0.5 * log_positions * (log_positions + 1.0) * (positions > 2048.0 ? positions / 2048.0 : 1.0);
    const double large_us = std::ceil(static_cast<double>(n) / kLargeMaxGrid) * (10.0 + 2.0 * steps + 1.5 * mean_hops + 0.4 * stages);
    return large_us < wave_us;
}
inline long long large_grid(long long n) { return n < kLargeMaxGrid ? (n > 0 ? n : 1) : kLargeMaxGrid; }
// bytes of the workgroups' staging areas (loads, then hops), 0 when the wavefront kernel serves
inline size_t large_stage_bytes(int64_t n, long long cap)
{
    if (!large_rows_possible(cap)) return 0;
    const size_t slots = static_cast<size_t>(large_grid(n)) * static_cast<size_t>(cap);
    return align_up(slots * sizeof(float)) + align_up(slots * sizeof(uint16_t));
}

template <int MODE>
grf_status launch_rows_large(const GraphView& gv, const WalkLaw& law, int n_walks, int f_len, int n_f, const float* f, int cap,
                             int32_t* row_ptr, int32_t* col_out, float* val_out, long long val_stride, const float* dphi,
                             float* df_part, unsigned char* stage, hipStream_t stream)
{
    const size_t lds = static_cast<size_t>(cap) * 6;
    if (lds > 64 * 1024)
        GRF_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&rows_large_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)));
    const long long grid = large_grid(gv.n);
    float* stage_load = reinterpret_cast<float*>(stage);
    uint16_t* stage_hop = reinterpret_cast<uint16_t*>(stage + align_up(static_cast<size_t>(grid) * cap * sizeof(float)));
    hipLaunchKernelGGL((rows_large_kernel<MODE>), dim3(static_cast<unsigned>(grid)), dim3(kLargeBlock), lds, stream, gv, law, n_walks, f_len, n_f, f,
                       cap, row_ptr, col_out, val_out, val_stride, dphi, df_part, stage_load, stage_hop);
    GRF_LAUNCH_CHECK("rows_large_kernel");
    return GRF_OK;
}

// df[x] = sum over nodes of df_part[node][x], x in [0, n_f * f_len): one workgroup per x, fixed order.
__global__ __launch_bounds__(256) void df_reduce_kernel(const float* __restrict__ df_part, long long n, int width, float* __restrict__ df)
{
    __shared__ float part[256];
    const int x = blockIdx.x;
    float acc = 0.0f;
    for (long long i = threadIdx.x; i < n; i += 256) acc += df_part[i * width + x];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (static_cast<int>(threadIdx.x) < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) df[x] = part[0];
}

// ------------------------------------------------------------------------------------ scan / fill
// Exclusive prefix sum by one workgroup of 1024 threads (the inputs are row, column or cell counts: a few hundred
// thousand elements at most in practice) over tiles of 1024 * PER elements, which the workgroup holds in registers.
// A wavefront owns 64 * PER consecutive elements of the tile and reads them in PER / 4 steps of one kilobyte, lane l
// taking the 16 bytes at 4 l of the step (coalesced; all steps' loads are requested at once: one memory round trip per
// tile, and the next tile's loads are requested before the current one is worked on).  Per step the lanes' sums are scanned across the wavefront and carried into
// the next step; the wavefronts' totals are scanned through LDS.  Sums are kept in 64 bits so that a total beyond int32
// is reported as such (outputs saturate).
template <int PER>
__global__ __launch_bounds__(1024) void scan_resident_kernel(int32_t* __restrict__ data, long long n, long long* __restrict__ total64)
{
    constexpr int STEPS = PER / 4;
    __shared__ long long wave_total[2][16];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const bool aligned = (reinterpret_cast<uintptr_t>(data) & 15u) == 0;
    auto saturated = [](long long x) { return x > 2147483647ll ? 2147483647 : static_cast<int32_t>(x); };
    long long carry = 0;
    int parity = 0;
    const long long in_tile = static_cast<long long>(wave) * (kWave * PER) + 4 * lane;
    auto load_tile = [&](long long tile, int32_t (&v)[STEPS][4]) {
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const long long idx = tile + in_tile + static_cast<long long>(j) * (4 * kWave);
            if (aligned && idx + 3 < n) {
                const int4 q = *reinterpret_cast<const int4*>(data + idx);
                v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) v[j][k] = (idx + k < n) ? data[idx + k] : 0;
            }
        }
    };
    int32_t v[STEPS][4], ahead[STEPS][4];
    load_tile(0, v);
    for (long long tile = 0; tile < n; tile += 1024ll * PER, parity ^= 1) {
        const long long base = tile + in_tile;
        // the next tile is requested before this one is worked on (its elements are not written by this tile's stores)
        if (tile + 1024ll * PER < n) load_tile(tile + 1024ll * PER, ahead);
        long long before_lane[STEPS];      // sum of the wavefront's elements that precede this lane's four of step j
        long long wave_sum = 0;
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const long long mine = static_cast<long long>(v[j][0]) + v[j][1] + v[j][2] + v[j][3];
            long long incl = mine;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const long long up = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += up;
            }
            before_lane[j] = wave_sum + incl - mine;
            wave_sum += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) wave_total[parity][wave] = wave_sum;
        __syncthreads();          // one barrier per tile: the two halves of wave_total alternate
        long long before = 0, tile_total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const long long t = wave_total[parity][w];
            if (w < wave) before += t;
            tile_total += t;
        }
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const long long idx = base + static_cast<long long>(j) * (4 * kWave);
            long long run = carry + before + before_lane[j];
            int32_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                o[k] = saturated(run);
                run += v[j][k];
            }
            if (aligned && idx + 3 < n) {
                *reinterpret_cast<int4*>(data + idx) = make_int4(o[0], o[1], o[2], o[3]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (idx + k < n) data[idx + k] = o[k];
            }
        }
        carry += tile_total;
#pragma unroll
        for (int j = 0; j < STEPS; ++j)
#pragma unroll
            for (int k = 0; k < 4; ++k) v[j][k] = ahead[j][k];
    }
    if (tid == 0) {
        data[n] = saturated(carry);
        if (total64 != nullptr) *total64 = carry;
    }
}

__global__ __launch_bounds__(256) void fill_kernel(int32_t* __restrict__ data, long long n, int32_t value)
{
    const long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) data[i] = value;
}

grf_status exclusive_scan_inplace(int32_t* counts, int64_t n, long long* total64, hipStream_t stream)
{
    const long long count = static_cast<long long>(n);
    hipLaunchKernelGGL(scan_resident_kernel<16>, dim3(1), dim3(1024), 0, stream, counts, count, total64);
    GRF_LAUNCH_CHECK("scan_resident_kernel");
    return GRF_OK;
}

grf_status fill_i32(int32_t* data, int64_t n, int32_t value, hipStream_t stream)
{
    if (n <= 0) return GRF_OK;
    const unsigned blocks = static_cast<unsigned>((n + 255) / 256);
    hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, stream, data, static_cast<long long>(n), value);
    GRF_LAUNCH_CHECK("fill_kernel");
    return GRF_OK;
}

// ------------------------------------------------------------------------------------ host side
namespace {


grf_status check_graph(const grf_graph* g)
{
    if (g == nullptr) return fail(GRF_EINVAL, "graph is NULL");
    if (g->n < 0 || g->nnz < 0) return fail(GRF_EINVAL, "graph n=%lld nnz=%lld must be >= 0", (long long)g->n, (long long)g->nnz);
    if (g->n >= 2147483647ll || g->nnz >= 2147483647ll) return fail(GRF_EUNSUPPORTED, "graph n and nnz must be < 2^31 - 1");
    if (g->row_ptr == nullptr) return fail(GRF_EINVAL, "graph row_ptr is NULL");
    if (g->nnz > 0 && (g->col == nullptr || g->w == nullptr)) return fail(GRF_EINVAL, "graph col / w is NULL");
    return GRF_OK;
}

grf_status make_law(double p_halt, uint64_t seed, WalkLaw* law)
{
    if (!(p_halt >= 0.0 && p_halt <= 1.0)) return fail(GRF_EINVAL, "p_halt=%g must lie in [0, 1]", p_halt);
    const double scaled = p_halt * 4294967296.0;
    const uint64_t thr = static_cast<uint64_t>(scaled);   // floor for non-negative values
    law->key0 = static_cast<uint32_t>(seed & 0xffffffffull);
    law->key1 = static_cast<uint32_t>(seed >> 32);
    law->always_halt = thr > 0xffffffffull ? 1 : 0;
    law->threshold = law->always_halt ? 0xffffffffu : static_cast<uint32_t>(thr);
    law->inv_survive = p_halt < 1.0 ? static_cast<float>(1.0 / (1.0 - p_halt)) : 0.0f;
    return GRF_OK;
}

GraphView view_of(const grf_graph* g)
{
    return GraphView{g->row_ptr, g->col, g->w, static_cast<int32_t>(g->n), static_cast<int32_t>(g->nnz)};
}

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" int64_t grf_sample_nnz_bound(int64_t n, int32_t n_walks, int32_t f_len)
{
    if (n < 0 || n_walks < 1 || f_len < 1) return -1;
    return n * (1 + static_cast<int64_t>(n_walks) * (f_len - 1));
}

extern "C" size_t grf_sample_workspace_bytes(int64_t n, int32_t n_walks, int32_t f_len, int32_t n_f)
{
    if (n < 0 || n_walks < 1 || f_len < 1 || n_f < 1) return 0;
    const long long cap = 1 + static_cast<long long>(n_walks) * (f_len - 1);
    return align_up(sizeof(float) * static_cast<size_t>(n_f) * f_len) + kAlign + large_stage_bytes(n, cap);
}

extern "C" grf_status grf_sample_walks(const grf_graph* g, double p_halt, int32_t n_walks, int32_t max_nodes,
                                       uint64_t seed, void* hip_stream, int32_t* traj)
{
    if (grf_status st = check_graph(g)) return st;
    if (n_walks < 1 || max_nodes < 1) return fail(GRF_EINVAL, "n_walks=%d and max_nodes=%d must be >= 1", n_walks, max_nodes);
    WalkLaw law;
    if (grf_status st = make_law(p_halt, seed, &law)) return st;
    if (g->n == 0) return GRF_OK;
    if (traj == nullptr) return fail(GRF_EINVAL, "traj is NULL");
    const long long total = static_cast<long long>(g->n) * n_walks;
    if (total * max_nodes >= (1ll << 40)) return fail(GRF_EUNSUPPORTED, "trajectory dump of %lld entries is too large", total * max_nodes);
    const long long blocks = (total + 255) / 256;
    if (blocks > 2147483647ll) return fail(GRF_EUNSUPPORTED, "too many walks for one launch");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(walks_kernel, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                       view_of(g), law, n_walks, max_nodes, traj);
    GRF_LAUNCH_CHECK("walks_kernel");
    return GRF_OK;
}

namespace {

// Both sampling entry points.  f_host: copied to the workspace first (else f_device is used in place).
// nnz_out: the stream is synchronised once to return the count (else capacity must cover the bound).
grf_status sample_impl(const grf_graph* g, const float* f_host, const float* f_device, int32_t f_len, int32_t n_f,
                       double p_halt, int32_t n_walks, uint64_t seed, void* workspace, size_t workspace_bytes,
                       hipStream_t stream, grf_phi* phi_out, int64_t* nnz_out)
{
    if (grf_status st = check_graph(g)) return st;
    if (f_host == nullptr && f_device == nullptr) return fail(GRF_EINVAL, "f is NULL");
    if (f_len < 1 || n_f < 1 || n_walks < 1)
        return fail(GRF_EINVAL, "f_len=%d, n_f=%d, n_walks=%d must all be >= 1", f_len, n_f, n_walks);
    if (f_len > 65535) return fail(GRF_EUNSUPPORTED, "f_len=%d exceeds 65535", f_len);
    WalkLaw law;
    if (grf_status st = make_law(p_halt, seed, &law)) return st;
    if (phi_out == nullptr) return fail(GRF_EINVAL, "phi_out is NULL");
    if (phi_out->n != g->n) return fail(GRF_EINVAL, "phi_out->n=%lld differs from graph n=%lld", (long long)phi_out->n, (long long)g->n);
    if (phi_out->row_ptr == nullptr) return fail(GRF_EINVAL, "phi_out->row_ptr is NULL");
    if (phi_out->capacity < 0) return fail(GRF_EINVAL, "phi_out->capacity is negative");
    if (phi_out->capacity > 0 && (phi_out->col == nullptr || phi_out->val == nullptr))
        return fail(GRF_EINVAL, "phi_out->col / val is NULL with capacity %lld", (long long)phi_out->capacity);
    const long long cap_ll = 1 + static_cast<long long>(n_walks) * (f_len - 1);
    if (cap_ll > kLargeMaxDeposits)
        return fail(GRF_EUNSUPPORTED, "1 + n_walks*(f_len-1) = %lld deposits per node exceed the %d that a workgroup orders in LDS", cap_ll, kLargeMaxDeposits);
    const size_t need = grf_sample_workspace_bytes(g->n, n_walks, f_len, n_f);
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return fail(GRF_EWORKSPACE, "workspace must be non-NULL, 256-byte aligned and >= %zu bytes (got %zu)", need, workspace_bytes);
    if (nnz_out == nullptr) {
        const int64_t bound = grf_sample_nnz_bound(g->n, n_walks, f_len);
        if (bound >= 2147483647ll) return fail(GRF_EUNSUPPORTED, "the bound n*(1+n_walks*(f_len-1)) = %lld must fit int32", (long long)bound);
        if (phi_out->capacity < bound)
            return fail(GRF_ECAPACITY, "phi_out->capacity must be at least grf_sample_nnz_bound() = %lld (got %lld)",
                        (long long)bound, (long long)phi_out->capacity);
    }

    unsigned char* ws = static_cast<unsigned char*>(workspace);
    long long* total_dev = reinterpret_cast<long long*>(ws + align_up(sizeof(float) * static_cast<size_t>(n_f) * f_len));
    if (g->n == 0) {
        if (grf_status st = fill_i32(phi_out->row_ptr, 1, 0, stream)) return st;
        if (nnz_out != nullptr) *nnz_out = 0;
        return GRF_OK;
    }
    const float* f_dev = f_device;
    if (f_host != nullptr) {
        GRF_HIP_TRY(hipMemcpyAsync(ws, f_host, sizeof(float) * static_cast<size_t>(n_f) * f_len, hipMemcpyHostToDevice, stream));
        f_dev = reinterpret_cast<const float*>(ws);
    }

    const int cap = static_cast<int>(cap_ll);
    const GraphView gv = view_of(g);

    // rows with many possible deposits: a workgroup per node, staging areas behind f and the counter
    const bool large = large_rows(g->n, cap_ll, n_walks, f_len, p_halt, kDepositBytes);
    unsigned char* stage = ws + align_up(sizeof(float) * static_cast<size_t>(n_f) * f_len) + kAlign;

    // pass 1: entries per row, then offsets
    if (grf_status st = large ? launch_rows_large<kCount>(gv, law, n_walks, f_len, n_f, f_dev, cap, phi_out->row_ptr, nullptr, nullptr, 0ll,
                                                          nullptr, nullptr, stage, stream)
                              : launch_rows<kCount>(gv, law, n_walks, f_len, n_f, f_dev, cap, phi_out->row_ptr, nullptr, nullptr, 0ll,
                                                    nullptr, nullptr, stream)) return st;
    if (grf_status st = exclusive_scan_inplace(phi_out->row_ptr, g->n, total_dev, stream)) return st;
    if (nnz_out != nullptr) {
        long long total = 0;
        GRF_HIP_TRY(hipMemcpyAsync(&total, total_dev, sizeof(long long), hipMemcpyDeviceToHost, stream));
        GRF_HIP_TRY(hipStreamSynchronize(stream));
        *nnz_out = total;
        if (total >= 2147483647ll) return fail(GRF_EUNSUPPORTED, "Phi_hat has %lld entries; int32 offsets cover < 2^31 - 1", total);
        if (phi_out->capacity < total)
            return fail(GRF_ECAPACITY, "Phi_hat has %lld entries but phi_out->capacity is %lld", total, (long long)phi_out->capacity);
    }

    // pass 2: same walks again, entries written at their offsets
    if (grf_status st = large ? launch_rows_large<kFill>(gv, law, n_walks, f_len, n_f, f_dev, cap, phi_out->row_ptr, phi_out->col, phi_out->val,
                                                         static_cast<long long>(phi_out->capacity), nullptr, nullptr, stage, stream)
                              : launch_rows<kFill>(gv, law, n_walks, f_len, n_f, f_dev, cap, phi_out->row_ptr, phi_out->col, phi_out->val,
                                                   static_cast<long long>(phi_out->capacity), nullptr, nullptr, stream)) return st;
    return GRF_OK;
}

}  // namespace

extern "C" grf_status grf_sample(const grf_graph* g, const float* f, int32_t f_len, int32_t n_f,
                                 double p_halt, int32_t n_walks, uint64_t seed,
                                 void* workspace, size_t workspace_bytes, void* hip_stream,
                                 grf_phi* phi_out, int64_t* nnz_out)
{
    if (grf_status st = check_graph(g)) return st;
    if (f == nullptr) return fail(GRF_EINVAL, "f is NULL");
    if (nnz_out == nullptr) return fail(GRF_EINVAL, "nnz_out is NULL");
    return sample_impl(g, f, nullptr, f_len, n_f, p_halt, n_walks, seed, workspace, workspace_bytes,
                       static_cast<hipStream_t>(hip_stream), phi_out, nnz_out);
}

extern "C" grf_status grf_sample_async(const grf_graph* g, const float* f_device, int32_t f_len, int32_t n_f,
                                       double p_halt, int32_t n_walks, uint64_t seed,
                                       void* workspace, size_t workspace_bytes, void* hip_stream, grf_phi* phi_out)
{
    if (grf_status st = check_graph(g)) return st;
    if (f_device == nullptr) return fail(GRF_EINVAL, "f_device is NULL");
    return sample_impl(g, nullptr, f_device, f_len, n_f, p_halt, n_walks, seed, workspace, workspace_bytes,
                       static_cast<hipStream_t>(hip_stream), phi_out, nullptr);
}

namespace {
size_t df_part_bytes(int64_t n, int32_t f_len, int32_t n_f)
{
    return align_up(sizeof(float) * static_cast<size_t>(n > 0 ? n : 1) * static_cast<size_t>(n_f) * static_cast<size_t>(f_len));
}
}  // namespace

extern "C" size_t grf_sample_backward_workspace_bytes(int64_t n, int32_t n_walks, int32_t f_len, int32_t n_f)
{
    if (n < 0 || n_walks < 1 || f_len < 1 || n_f < 1) return 0;
    const long long cap = 1 + static_cast<long long>(n_walks) * (f_len - 1);
    return df_part_bytes(n, f_len, n_f) + large_stage_bytes(n, cap);
}

extern "C" grf_status grf_sample_backward(const grf_graph* g, int32_t f_len, int32_t n_f,
                                          double p_halt, int32_t n_walks, uint64_t seed,
                                          const grf_phi* phi, int64_t nnz, const float* dphi_val,
                                          void* workspace, size_t workspace_bytes, void* hip_stream, float* df)
{
    if (grf_status st = check_graph(g)) return st;
    if (f_len < 1 || n_f < 1 || n_walks < 1)
        return fail(GRF_EINVAL, "f_len=%d, n_f=%d, n_walks=%d must all be >= 1", f_len, n_f, n_walks);
    if (f_len > 65535) return fail(GRF_EUNSUPPORTED, "f_len=%d exceeds 65535", f_len);
    WalkLaw law;
    if (grf_status st = make_law(p_halt, seed, &law)) return st;
    if (phi == nullptr || df == nullptr) return fail(GRF_EINVAL, "phi / df is NULL");
    if (phi->n != g->n) return fail(GRF_EINVAL, "phi->n=%lld differs from graph n=%lld", (long long)phi->n, (long long)g->n);
    if (nnz < 0 || nnz > phi->capacity || nnz >= 2147483647ll) return fail(GRF_EINVAL, "nnz=%lld must lie in [0, phi->capacity=%lld]", (long long)nnz, (long long)phi->capacity);
    if (phi->row_ptr == nullptr || (nnz > 0 && dphi_val == nullptr)) return fail(GRF_EINVAL, "phi->row_ptr / dphi_val is NULL");
    const long long cap_ll = 1 + static_cast<long long>(n_walks) * (f_len - 1);
    if (cap_ll > kLargeMaxDeposits)
        return fail(GRF_EUNSUPPORTED, "1 + n_walks*(f_len-1) = %lld deposits per node exceed the %d that a workgroup orders in LDS", cap_ll, kLargeMaxDeposits);
    const size_t need = grf_sample_backward_workspace_bytes(g->n, n_walks, f_len, n_f);
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return fail(GRF_EWORKSPACE, "workspace must be non-NULL, 256-byte aligned and >= %zu bytes (got %zu)", need, workspace_bytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int width = n_f * f_len;
    if (g->n == 0) {
        if (grf_status st = fill_i32(reinterpret_cast<int32_t*>(df), width, 0, stream)) return st;
        return GRF_OK;
    }
    float* df_part = static_cast<float*>(workspace);
    const int cap = static_cast<int>(cap_ll);
    unsigned char* stage = static_cast<unsigned char*>(workspace) + df_part_bytes(g->n, f_len, n_f);
    if (grf_status st = large_rows(g->n, cap_ll, n_walks, f_len, p_halt, kDepositBytesGrad) ? launch_rows_large<kGrad>(view_of(g), law, n_walks, f_len, n_f, nullptr, cap, phi->row_ptr, nullptr, nullptr,
                                                                      static_cast<long long>(phi->capacity), dphi_val, df_part, stage, stream)
                                           : launch_rows<kGrad>(view_of(g), law, n_walks, f_len, n_f, nullptr, cap, phi->row_ptr, nullptr, nullptr,
                                                                static_cast<long long>(phi->capacity), dphi_val, df_part, stream)) return st;
    hipLaunchKernelGGL(df_reduce_kernel, dim3(static_cast<unsigned>(width)), dim3(256), 0, stream,
                       static_cast<const float*>(df_part), static_cast<long long>(g->n), width, df);
    GRF_LAUNCH_CHECK("df_reduce_kernel");
    return GRF_OK;
}

extern "C" void grf_debug_force_row_kernel(int32_t which)
{
    g_force_row_kernel.store(which >= 1 && which <= 3 ? which : 0, std::memory_order_relaxed);
}
