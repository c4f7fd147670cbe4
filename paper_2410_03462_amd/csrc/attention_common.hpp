// Pieces shared by the attention translation units: element loads, the column lists of
// Phi_hat (who contributes to / consumes bucket l) and host-side argument checks.
#pragma once

#include "common.hpp"

namespace grf {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(static_cast<uint32_t>(x.bits) << 16); }

__device__ __forceinline__ float feature(float x, int relu) { return relu ? fmaxf(x, 0.0f) : x; }

// Column lists of Phi_hat, carved out of the caller's workspace.
struct Transposed {
    int32_t* col_ptr;   // [n+1]
    int32_t* cursor;    // [n]
    int32_t* u_row;     // [nnz] unsorted
    int32_t* u_src;
    int32_t* s_row;     // [nnz] rows ascending inside each column
    int32_t* s_src;     // index of the entry in CSR order (addresses every value plane)
    int32_t* csr_to_csc;  // [nnz] position in the column lists of CSR entry e
    long long* total;
    size_t bytes;
};

Transposed carve_transposed(unsigned char* ws, int64_t n, int64_t nnz);
grf_status transpose(const grf_phi* phi, int64_t nnz, const Transposed& t, hipStream_t stream);
grf_status check_problem(const void* a, const void* b, int32_t dtype, int64_t B, int64_t H, int64_t n, int32_t d,
                         const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map);
grf_status check_workspace(const void* workspace, size_t have, size_t need);

inline unsigned blocks_for(long long items, int per_block) { return static_cast<unsigned>((items + per_block - 1) / per_block); }

// Dispatch on (d, dtype) to the compiled instances.
#define GRF_DISPATCH(d, dtype, CALL)                                                     \
    do {                                                                                 \
        if ((d) == 64 && (dtype) == GRF_DTYPE_F32) { constexpr int D_ = 64; using T_ = float; CALL; }  \
        else if ((d) == 64) { constexpr int D_ = 64; using T_ = bf16_t; CALL; }          \
        else if ((dtype) == GRF_DTYPE_F32) { constexpr int D_ = 32; using T_ = float; CALL; }          \
        else { constexpr int D_ = 32; using T_ = bf16_t; CALL; }                         \
    } while (0)

}  // namespace grf
