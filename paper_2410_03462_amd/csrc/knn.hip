// k-nearest-neighbour graph of a 3-D point cloud, built on the GPU.
//
// For dynamic point clouds the graph changes at every step, the walks cannot be precomputed and
// the paper names the neighbour search as the bottleneck of that setting (Sec. 4, point-cloud
// experiment; App. C).  The paper uses an unspecified approximate solver; this one is exact:
//
//   1. bounding box, then a uniform grid with about one point per two cells (device-side, no host sync);
//   2. counting sort of the points by cell (histogram, scan, scatter);
//   3. eight lanes per query point, queries in cell order: cells are visited in shells of growing Chebyshev
//      radius around the query's cell and the k best (squared distance, index) pairs are kept in
//      registers; the search stops when the k-th best distance is below the distance to anything
//      outside the visited shells;
//   4. assembly of the CSR graph: directed lists, or their symmetric closure (i ~ j if either lists
//      the other), columns ascending, weights from the distances, rows normalised.
//
// Squared distances are taken in fp32 with a fixed operation order and no fused multiply-adds, and
// ties are broken by the smaller index, so the neighbour lists are a pure function of the
// coordinates (they do not depend on the grid or on scheduling).
#include "common.hpp"

namespace grf {

namespace {
constexpr int kMaxGridDim = 256;
constexpr float kTargetPerCell = 0.5f;      // mean points per cell: small cells keep the shells tight where the cloud is dense
}  // namespace

struct KnnGrid {
    float lo[3];
    float inv_h;
    float h;
    int dims[3];
    int cells;
};

// fl(fl(fl(dx dx) + fl(dy dy)) + fl(dz dz)) with dx = fl(a.x - b.x): every operation rounded on its own.
// (Contraction into fused multiply-adds is switched off for this block: the products must be rounded.)
__device__ __forceinline__ float squared_distance(float ax, float ay, float az, float bx, float by, float bz)
{
#pragma clang fp contract(off)
    const float dx = ax - bx, dy = ay - by, dz = az - bz;
    const float xx = dx * dx, yy = dy * dy, zz = dz * dz;
    const float xy = xx + yy;
    return xy + zz;
}

__device__ __forceinline__ int cell_coordinate(float x, float lo, float inv_h, int dim)
{
    const int c = static_cast<int>(floorf((x - lo) * inv_h));
    return min(max(c, 0), dim - 1);
}

// ------------------------------------------------------------------------------------ grid
// One workgroup: bounding box by a tree reduction, then the cell size: the largest g <= kMaxGridDim such that
// a cell of edge (largest extent / g) gives at most n / kTargetPerCell cells.
__global__ __launch_bounds__(1024) void knn_grid_kernel(const float* __restrict__ pts, long long n, KnnGrid* __restrict__ grid)
{
    __shared__ float smin[3][1024], smax[3][1024];
    const int tid = threadIdx.x;
    float mn[3] = {__builtin_inff(), __builtin_inff(), __builtin_inff()};
    float mx[3] = {-__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
    for (long long i = tid; i < n; i += 1024)
        for (int a = 0; a < 3; ++a) {
            const float v = pts[3 * i + a];
            mn[a] = fminf(mn[a], v);
            mx[a] = fmaxf(mx[a], v);
        }
    for (int a = 0; a < 3; ++a) { smin[a][tid] = mn[a]; smax[a][tid] = mx[a]; }
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if (tid < off)
            for (int a = 0; a < 3; ++a) {
                smin[a][tid] = fminf(smin[a][tid], smin[a][tid + off]);
                smax[a][tid] = fmaxf(smax[a][tid], smax[a][tid + off]);
            }
        __syncthreads();
    }
    if (tid == 0) {
        float ext[3], big = 0.0f;
        for (int a = 0; a < 3; ++a) { ext[a] = smax[a][0] - smin[a][0]; big = fmaxf(big, ext[a]); }
        const long long budget = max(1ll, static_cast<long long>(static_cast<float>(n) / kTargetPerCell));
        int best = 1;
        if (big > 0.0f && isfinite(big)) {
            int lo_g = 1, hi_g = kMaxGridDim;
            while (lo_g <= hi_g) {
                const int g = (lo_g + hi_g) / 2;
                const float h = big / static_cast<float>(g);
                long long cells = 1;
                for (int a = 0; a < 3; ++a) cells *= max(1, min(g, static_cast<int>(ceilf(ext[a] / h))));
                if (cells <= budget) { best = g; lo_g = g + 1; } else { hi_g = g - 1; }
            }
        }
        const float h = (big > 0.0f && isfinite(big)) ? big / static_cast<float>(best) : 1.0f;
        int cells = 1;
        for (int a = 0; a < 3; ++a) {
            grid->lo[a] = smin[a][0];
            grid->dims[a] = (big > 0.0f && isfinite(big)) ? max(1, min(best, static_cast<int>(ceilf(ext[a] / h)))) : 1;
            cells *= grid->dims[a];
        }
        grid->h = h;
        grid->inv_h = 1.0f / h;
        grid->cells = cells;
    }
}

__device__ __forceinline__ int cell_of(const KnnGrid& g, float x, float y, float z)
{
    const int cx = cell_coordinate(x, g.lo[0], g.inv_h, g.dims[0]);
    const int cy = cell_coordinate(y, g.lo[1], g.inv_h, g.dims[1]);
    const int cz = cell_coordinate(z, g.lo[2], g.inv_h, g.dims[2]);
    return (cz * g.dims[1] + cy) * g.dims[0] + cx;
}

__global__ __launch_bounds__(256) void knn_cell_count_kernel(const float* __restrict__ pts, long long n, const KnnGrid* __restrict__ grid,
                                                             int32_t* __restrict__ cell_of_point, int32_t* __restrict__ cell_count)
{
    const long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const KnnGrid g = *grid;
    const int c = cell_of(g, pts[3 * i], pts[3 * i + 1], pts[3 * i + 2]);
    cell_of_point[i] = c;
    atomicAdd(&cell_count[c], 1);
}

// sorted[pos] = (x, y, z, index bits); the order inside a cell depends on atomic arrival, which the
// search does not care about (its result is a function of the set of candidates).
__global__ __launch_bounds__(256) void knn_cell_scatter_kernel(const float* __restrict__ pts, long long n,
                                                               const int32_t* __restrict__ cell_of_point,
                                                               const int32_t* __restrict__ cell_start, int32_t* __restrict__ cursor,
                                                               float4* __restrict__ sorted)
{
    const long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int c = cell_of_point[i];
    const int pos = cell_start[c] + atomicAdd(&cursor[c], 1);
    sorted[pos] = make_float4(pts[3 * i], pts[3 * i + 1], pts[3 * i + 2], __int_as_float(static_cast<int>(i)));
}

// ------------------------------------------------------------------------------------ search
// Eight lanes per query point (eight queries per wavefront), queries in cell order.  The cells of a shell are
// scanned as runs of consecutive points (a row of cells along x is one run in the sorted array); the eight
// lanes take eight points of a run at a time, and those that beat the current k-th best are inserted one
// after the other into the list, which every lane of the group holds (sorted ascending by (distance, index);
// unused slots hold (+inf, INT_MAX)).
constexpr int kLanesPerQuery = 8;

template <int KMAX>
__global__ __launch_bounds__(64) void knn_search_kernel(const float4* __restrict__ sorted, long long n, int k,
                                                         const KnnGrid* __restrict__ grid, const int32_t* __restrict__ cell_start,
                                                         int32_t* __restrict__ knn_idx, float* __restrict__ knn_d2)
{
    constexpr int L = kLanesPerQuery;
    const int lane = lane_id();
    const int sub = lane % L;                         // lane inside the group
    const int group_base = lane - sub;                // first lane of the group
    const long long t = (static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x) / L;
    if (t >= n) return;                               // whole groups leave together
    const KnnGrid g = *grid;
    const float4 me = sorted[t];
    const int my_index = __float_as_int(me.w);
    const int cx = cell_coordinate(me.x, g.lo[0], g.inv_h, g.dims[0]);
    const int cy = cell_coordinate(me.y, g.lo[1], g.inv_h, g.dims[1]);
    const int cz = cell_coordinate(me.z, g.lo[2], g.inv_h, g.dims[2]);

    float bd[KMAX];
    int bi[KMAX];
#pragma unroll
    for (int s = 0; s < KMAX; ++s) { bd[s] = __builtin_inff(); bi[s] = 2147483647; }
    float worst_d = __builtin_inff();       // slot k - 1
    int worst_i = 2147483647;

    // points [beg, end) of the sorted array
    auto visit_run = [&](int beg, int end) {
        for (int p0 = beg; p0 < end; p0 += L) {
            const int p = p0 + sub;
            const float4 q = sorted[min(p, end - 1)];
            const int j = __float_as_int(q.w);
            const float d = squared_distance(me.x, me.y, me.z, q.x, q.y, q.z);
            const bool pass = p < end && j != my_index && (d < worst_d || (d == worst_d && j < worst_i));
            unsigned pending = static_cast<unsigned>(__ballot(pass) >> group_base) & ((1u << L) - 1u);
            while (pending != 0u) {
                const int src = group_base + __builtin_ctz(pending);
                pending &= pending - 1u;
                float cd = __shfl(d, src, kWave);
                int ci = __shfl(j, src, kWave);
                if (!(cd < worst_d || (cd == worst_d && ci < worst_i))) continue;      // the list has moved on
#pragma unroll
                for (int s = 0; s < KMAX; ++s) {
                    const bool less = (cd < bd[s]) || (cd == bd[s] && ci < bi[s]);
                    const float td = less ? bd[s] : cd;
                    const int ti = less ? bi[s] : ci;
                    bd[s] = less ? cd : bd[s];
                    bi[s] = less ? ci : bi[s];
                    cd = td; ci = ti;
                }
#pragma unroll
                for (int s = 0; s < KMAX; ++s)
                    if (s == k - 1) { worst_d = bd[s]; worst_i = bi[s]; }
            }
        }
    };
    auto visit_cells = [&](int x0, int x1, int y, int z) {      // cells x0 .. x1 of row (y, z): one run
        const int c0 = (z * g.dims[1] + y) * g.dims[0];
        visit_run(cell_start[c0 + x0], cell_start[c0 + x1 + 1]);
    };

    const int max_ring = max(g.dims[0], max(g.dims[1], g.dims[2]));
    const int cc[3] = {cx, cy, cz};
    const float mp[3] = {me.x, me.y, me.z};
    for (int r = 0; r <= max_ring; ++r) {
        if (r > 0) {
            // shells 0 .. r-1 cover the box of cells [c - (r-1), c + (r-1)] on every axis; whatever is outside is at
            // least as far as the nearest face of that box that still has cells beyond it.  A margin of 0.01 cell
            // edges covers the rounding of the cell coordinates.
            float reach = __builtin_inff();
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                const float rel = (mp[a] - g.lo[a]) * g.inv_h;       // query position in cell units
                if (cc[a] - (r - 1) > 0) reach = fminf(reach, rel - static_cast<float>(cc[a] - (r - 1)));
                if (cc[a] + (r - 1) < g.dims[a] - 1) reach = fminf(reach, static_cast<float>(cc[a] + r) - rel);
            }
            if (reach == __builtin_inff()) break;                    // every cell has been visited
            reach = (reach - 0.01f) * g.h;
            if (reach > 0.0f && worst_d <= reach * reach) break;
        }
        const int z0 = max(cz - r, 0), z1 = min(cz + r, g.dims[2] - 1);
        const int y0 = max(cy - r, 0), y1 = min(cy + r, g.dims[1] - 1);
        const int x0 = max(cx - r, 0), x1 = min(cx + r, g.dims[0] - 1);
        for (int z = z0; z <= z1; ++z) {
            const bool zface = (z == cz - r) || (z == cz + r);
            for (int y = y0; y <= y1; ++y) {
                const bool face = zface || (y == cy - r) || (y == cy + r);
                if (face) {
                    visit_cells(x0, x1, y, z);
                } else {
                    if (cx - r >= 0) visit_cells(cx - r, cx - r, y, z);
                    if (cx + r < g.dims[0]) visit_cells(cx + r, cx + r, y, z);
                }
            }
        }
    }
    if (sub == 0) {
#pragma unroll
        for (int s = 0; s < KMAX; ++s)
            if (s < k) {
                knn_idx[static_cast<long long>(my_index) * k + s] = bi[s] == 2147483647 ? -1 : bi[s];
                knn_d2[static_cast<long long>(my_index) * k + s] = bd[s];
            }
    }
}

// ------------------------------------------------------------------------------------ graph assembly
// Entries of row i: its own list, plus, when symmetrising, every j that lists i without being listed by i.
__global__ __launch_bounds__(256) void knn_degree_kernel(const int32_t* __restrict__ knn_idx, long long n, int k, int symmetrise,
                                                         int32_t* __restrict__ degree)
{
    const long long e = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= n * k) return;
    const long long i = e / k;
    const int32_t j = knn_idx[e];
    if (j < 0) return;
    atomicAdd(&degree[i], 1);
    if (symmetrise) {
        bool mutual = false;
        for (int s = 0; s < k; ++s) mutual |= knn_idx[static_cast<long long>(j) * k + s] == static_cast<int32_t>(i);
        if (!mutual) atomicAdd(&degree[j], 1);
    }
}

__global__ __launch_bounds__(256) void knn_edges_kernel(const int32_t* __restrict__ knn_idx, const float* __restrict__ knn_d2,
                                                        long long n, int k, int symmetrise, const int32_t* __restrict__ row_ptr,
                                                        int32_t* __restrict__ cursor, int32_t* __restrict__ u_col, float* __restrict__ u_d2)
{
    const long long e = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= n * k) return;
    const long long i = e / k;
    const int32_t j = knn_idx[e];
    if (j < 0) return;
    const float d2 = knn_d2[e];
    int slot = row_ptr[i] + atomicAdd(&cursor[i], 1);
    u_col[slot] = j; u_d2[slot] = d2;
    if (symmetrise) {
        bool mutual = false;
        for (int s = 0; s < k; ++s) mutual |= knn_idx[static_cast<long long>(j) * k + s] == static_cast<int32_t>(i);
        if (!mutual) {
            slot = row_ptr[j] + atomicAdd(&cursor[j], 1);
            u_col[slot] = static_cast<int32_t>(i); u_d2[slot] = d2;
        }
    }
}

// One wavefront per row: columns ranked by counting (distinct within a row) and unnormalised weights from the
// distances.  weight_kind: GRF_WEIGHT_INV_DEGREE, GRF_WEIGHT_EXP = exp(-dist/sigma), GRF_WEIGHT_GAUSS = exp(-dist^2/(2 sigma^2)).
__global__ __launch_bounds__(256) void knn_rows_kernel(const int32_t* __restrict__ row_ptr, long long n, const int32_t* __restrict__ u_col,
                                                       const float* __restrict__ u_d2, int weight_kind, float sigma,
                                                       int32_t* __restrict__ col, float* __restrict__ w)
{
    const long long i = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (i >= n) return;
    const int lane = lane_id();
    const int32_t beg = row_ptr[i];
    const int len = row_ptr[i + 1] - beg;
    // kernel weights are taken relative to the row's nearest neighbour (the factor cancels in the normalisation),
    // so that a row far from everything does not underflow to 0 / 0
    float nearest = __builtin_inff();
    for (int s = lane; s < len; s += kWave) nearest = fminf(nearest, u_d2[beg + s]);
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) nearest = fminf(nearest, __shfl_xor(nearest, off, kWave));
    for (int s = lane; s < len; s += kWave) {
        const int32_t key = u_col[beg + s];
        int rank = 0;
        for (int s2 = 0; s2 < len; ++s2) rank += static_cast<int>(u_col[beg + s2] < key);
        const float d2 = u_d2[beg + s];
        float raw = 1.0f;
        // the difference of two square roots in fp64: in fp32 its rounding error, divided by a small sigma, would
        // reach the weights of rows whose neighbours are far away
        if (weight_kind == GRF_WEIGHT_EXP)
            raw = expf(static_cast<float>(-(sqrt(static_cast<double>(d2)) - sqrt(static_cast<double>(nearest))) / static_cast<double>(sigma)));
        if (weight_kind == GRF_WEIGHT_GAUSS) raw = expf(-(d2 - nearest) / (2.0f * sigma * sigma));
        col[beg + rank] = key;
        w[beg + rank] = raw;
    }
}

// One wavefront per row: divide by the row sum, taken over the entries in their final (column) order so that
// it does not depend on the order in which the edges arrived.
__global__ __launch_bounds__(256) void knn_normalise_kernel(const int32_t* __restrict__ row_ptr, long long n, float* __restrict__ w)
{
    const long long i = static_cast<long long>(blockIdx.x) * (blockDim.x / kWave) + (threadIdx.x / kWave);
    if (i >= n) return;
    const int lane = lane_id();
    const int32_t beg = row_ptr[i];
    const int len = row_ptr[i + 1] - beg;
    float total = 0.0f;
    for (int s = lane; s < len; s += kWave) total += w[beg + s];
    total = wave_sum(total);
    for (int s = lane; s < len; s += kWave) w[beg + s] = w[beg + s] / total;
}

namespace {

struct KnnScratch {
    KnnGrid* grid;
    long long* total;
    int32_t* cell_of_point;   // [n]
    int32_t* cell_start;      // [cells + 2], cells <= 2 n
    int32_t* cursor;          // [2 n + 1]  (cells, then rows)
    float4* sorted;           // [n]
    int32_t* knn_idx;         // [n][k]
    float* knn_d2;            // [n][k]
    int32_t* u_col;           // [2 n k]
    float* u_d2;              // [2 n k]
    size_t bytes;
};

KnnScratch carve_knn(unsigned char* ws, int64_t n, int32_t k)
{
    KnnScratch s;
    size_t off = 0;
    auto take = [&](size_t bytes) { unsigned char* p = ws ? ws + off : nullptr; off += align_up(bytes); return p; };
    const size_t rows = static_cast<size_t>(n > 0 ? n : 1), kk = static_cast<size_t>(k > 0 ? k : 1);
    s.grid = reinterpret_cast<KnnGrid*>(take(sizeof(KnnGrid)));
    s.total = reinterpret_cast<long long*>(take(sizeof(long long)));
    s.cell_of_point = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * rows));
    s.cell_start = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (2 * rows + 2)));
    s.cursor = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (2 * rows + 1)));
    s.sorted = reinterpret_cast<float4*>(take(sizeof(float4) * rows));
    s.knn_idx = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * rows * kk));
    s.knn_d2 = reinterpret_cast<float*>(take(sizeof(float) * rows * kk));
    s.u_col = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * 2 * rows * kk));
    s.u_d2 = reinterpret_cast<float*>(take(sizeof(float) * 2 * rows * kk));
    s.bytes = off;
    return s;
}

constexpr int kMaxK = 32;

}  // namespace
}  // namespace grf

using namespace grf;

extern "C" int64_t grf_knn_graph_nnz_bound(int64_t n, int32_t k, int32_t symmetrise)
{
    if (n < 0 || k < 1 || k > kMaxK) return -1;
    return (symmetrise ? 2 : 1) * n * static_cast<int64_t>(k);
}

extern "C" size_t grf_knn_graph_workspace_bytes(int64_t n, int32_t k)
{
    if (n < 0 || k < 1 || k > kMaxK) return 0;
    return carve_knn(nullptr, n, k).bytes;
}

extern "C" grf_status grf_knn_graph(const float* points, int64_t n, int32_t k, int32_t symmetrise, int32_t weight_kind, float sigma,
                                    void* workspace, size_t workspace_bytes, void* hip_stream,
                                    int32_t* row_ptr, int32_t* col, float* w, int64_t capacity, int64_t* nnz_out)
{
    if (n < 0) return fail(GRF_EINVAL, "n=%lld must be >= 0", (long long)n);
    if (k < 1) return fail(GRF_EINVAL, "k=%d must be >= 1", k);
    if (k > kMaxK) return fail(GRF_EUNSUPPORTED, "k=%d exceeds %d", k, kMaxK);
    if (n * static_cast<int64_t>(k) >= (1ll << 30)) return fail(GRF_EUNSUPPORTED, "n*k=%lld is too large", (long long)(n * k));
    if (weight_kind != GRF_WEIGHT_INV_DEGREE && weight_kind != GRF_WEIGHT_EXP && weight_kind != GRF_WEIGHT_GAUSS)
        return fail(GRF_EINVAL, "weight_kind=%d is unknown", weight_kind);
    if (weight_kind != GRF_WEIGHT_INV_DEGREE && !(sigma > 0.0f)) return fail(GRF_EINVAL, "sigma=%g must be > 0", (double)sigma);
    if (row_ptr == nullptr) return fail(GRF_EINVAL, "row_ptr is NULL");
    if (nnz_out == nullptr && capacity < grf_knn_graph_nnz_bound(n, k, symmetrise))
        return fail(GRF_ECAPACITY, "without nnz_out capacity must be at least grf_knn_graph_nnz_bound() = %lld (got %lld)",
                    (long long)grf_knn_graph_nnz_bound(n, k, symmetrise), (long long)capacity);
    if (n > 0 && points == nullptr) return fail(GRF_EINVAL, "points is NULL");
    if (capacity < 0 || (capacity > 0 && (col == nullptr || w == nullptr))) return fail(GRF_EINVAL, "col / w is NULL or capacity < 0");
    const size_t need = grf_knn_graph_workspace_bytes(n, k);
    if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return fail(GRF_EWORKSPACE, "workspace must be non-NULL, 256-byte aligned and >= %zu bytes (got %zu)", need, workspace_bytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (n == 0) {
        if (grf_status st = fill_i32(row_ptr, 1, 0, stream)) return st;
        if (nnz_out != nullptr) *nnz_out = 0;
        return GRF_OK;
    }
    const KnnScratch s = carve_knn(static_cast<unsigned char*>(workspace), n, k);
    const unsigned pblocks = static_cast<unsigned>((n + 255) / 256);
    const unsigned eblocks = static_cast<unsigned>((n * k + 255) / 256);
    const unsigned sblocks = static_cast<unsigned>((n + 7) / 8);        // one wavefront = eight queries per workgroup: the searches differ in length

    hipLaunchKernelGGL(knn_grid_kernel, dim3(1), dim3(1024), 0, stream, points, static_cast<long long>(n), s.grid);
    GRF_LAUNCH_CHECK("knn_grid_kernel");
    if (grf_status st = fill_i32(s.cell_start, 2 * n + 2, 0, stream)) return st;
    if (grf_status st = fill_i32(s.cursor, 2 * n + 1, 0, stream)) return st;
    hipLaunchKernelGGL(knn_cell_count_kernel, dim3(pblocks), dim3(256), 0, stream, points, static_cast<long long>(n),
                       static_cast<const KnnGrid*>(s.grid), s.cell_of_point, s.cell_start);
    GRF_LAUNCH_CHECK("knn_cell_count_kernel");
    if (grf_status st = exclusive_scan_inplace(s.cell_start, 2 * n + 1, s.total, stream)) return st;     // cells <= 2 n
    hipLaunchKernelGGL(knn_cell_scatter_kernel, dim3(pblocks), dim3(256), 0, stream, points, static_cast<long long>(n),
                       static_cast<const int32_t*>(s.cell_of_point), static_cast<const int32_t*>(s.cell_start), s.cursor, s.sorted);
    GRF_LAUNCH_CHECK("knn_cell_scatter_kernel");

    const float4* sorted = s.sorted;
    const KnnGrid* grid = s.grid;
    const int32_t* cell_start = s.cell_start;
    if (k <= 4)
        hipLaunchKernelGGL((knn_search_kernel<4>), dim3(sblocks), dim3(64), 0, stream, sorted, static_cast<long long>(n), k, grid, cell_start, s.knn_idx, s.knn_d2);
    else if (k <= 8)
        hipLaunchKernelGGL((knn_search_kernel<8>), dim3(sblocks), dim3(64), 0, stream, sorted, static_cast<long long>(n), k, grid, cell_start, s.knn_idx, s.knn_d2);
    else if (k <= 16)
        hipLaunchKernelGGL((knn_search_kernel<16>), dim3(sblocks), dim3(64), 0, stream, sorted, static_cast<long long>(n), k, grid, cell_start, s.knn_idx, s.knn_d2);
    else
        hipLaunchKernelGGL((knn_search_kernel<32>), dim3(sblocks), dim3(64), 0, stream, sorted, static_cast<long long>(n), k, grid, cell_start, s.knn_idx, s.knn_d2);
    GRF_LAUNCH_CHECK("knn_search_kernel");

    // rows: degrees, offsets, edges, then ordered columns and weights
    if (grf_status st = fill_i32(row_ptr, n + 1, 0, stream)) return st;
    if (grf_status st = fill_i32(s.cursor, n + 1, 0, stream)) return st;
    hipLaunchKernelGGL(knn_degree_kernel, dim3(eblocks), dim3(256), 0, stream, static_cast<const int32_t*>(s.knn_idx),
                       static_cast<long long>(n), k, symmetrise ? 1 : 0, row_ptr);
    GRF_LAUNCH_CHECK("knn_degree_kernel");
    if (grf_status st = exclusive_scan_inplace(row_ptr, n, s.total, stream)) return st;
    if (nnz_out != nullptr) {
        long long total = 0;
        GRF_HIP_TRY(hipMemcpyAsync(&total, s.total, sizeof(long long), hipMemcpyDeviceToHost, stream));
        GRF_HIP_TRY(hipStreamSynchronize(stream));
        *nnz_out = total;
        if (capacity < total) return fail(GRF_ECAPACITY, "the graph has %lld entries but capacity is %lld", total, (long long)capacity);
    }
    hipLaunchKernelGGL(knn_edges_kernel, dim3(eblocks), dim3(256), 0, stream, static_cast<const int32_t*>(s.knn_idx),
                       static_cast<const float*>(s.knn_d2), static_cast<long long>(n), k, symmetrise ? 1 : 0,
                       static_cast<const int32_t*>(row_ptr), s.cursor, s.u_col, s.u_d2);
    GRF_LAUNCH_CHECK("knn_edges_kernel");
    hipLaunchKernelGGL(knn_rows_kernel, dim3(static_cast<unsigned>((n + 3) / 4)), dim3(256), 0, stream,
                       static_cast<const int32_t*>(row_ptr), static_cast<long long>(n), static_cast<const int32_t*>(s.u_col),
                       static_cast<const float*>(s.u_d2), weight_kind, sigma, col, w);
    GRF_LAUNCH_CHECK("knn_rows_kernel");
    hipLaunchKernelGGL(knn_normalise_kernel, dim3(static_cast<unsigned>((n + 3) / 4)), dim3(256), 0, stream,
                       static_cast<const int32_t*>(row_ptr), static_cast<long long>(n), w);
    GRF_LAUNCH_CHECK("knn_normalise_kernel");
    return GRF_OK;
}
