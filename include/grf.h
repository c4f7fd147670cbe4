/*
 * grf.h -- C ABI of the MI355X (gfx950) library for topologically masked linear attention
 * with graph random features (GRFs), after arXiv 2410.03462.
 *
 * The library does two things, both on one GPU and entirely in hand-written HIP kernels:
 *
 *   grf_sample                    graph (CSR) + modulation f + p_halt + n_walks + seed  ->  Phi_hat (CSR)
 *                                 [Sec. 3.3, GRF definition; Alg. 1 steps 1-2]
 *   grf_masked_linear_attention   Q, K, V, Phi_hat  ->  out = D^-1 (Phi_Q,G (Phi_K,G^T V))
 *                                 [Eq. 7 / Alg. 1 steps 3-5]
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer owned by the caller unless its comment says HOST.
 *     The library never allocates or frees device memory and keeps no state between calls; all
 *     temporaries live in the caller's workspace.
 *   - All work is enqueued on the caller's stream (a hipStream_t passed as void*; NULL is the
 *     default stream).  Two calls block on the stream, once each, to return a count to the host: grf_sample (nnz)
 *     and grf_knn_graph when nnz_out is given; grf_sample_async and grf_knn_graph with nnz_out == NULL do not.
 *   - Every entry point returns GRF_OK (0) or a negative grf_status; the message of the last error
 *     on the calling thread is available from grf_last_error().  Arguments are validated on the
 *     host before anything is launched; on error nothing partial is promised in the outputs.
 *   - Calls that share a workspace or an output buffer must not overlap in time.
 */
#ifndef GRF_H_
#define GRF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t grf_status;
#define GRF_OK            0
#define GRF_EINVAL       (-1)   /* an argument is out of its documented range, or a required pointer is NULL   */
#define GRF_ECAPACITY    (-2)   /* phi_out->capacity is smaller than the number of entries sampled             */
#define GRF_EUNSUPPORTED (-3)   /* valid request outside what the kernels cover (head dim, n_walks*f_len, nnz) */
#define GRF_EHIP         (-4)   /* a HIP runtime call or kernel launch reported an error                       */
#define GRF_EWORKSPACE   (-5)   /* workspace is NULL, misaligned (256 B) or smaller than *_workspace_bytes()   */

/* Element type of Q, K, V. */
#define GRF_DTYPE_F32   0
#define GRF_DTYPE_BF16  1       /* bfloat16 inputs; buckets, accumulation and outputs stay fp32 */

/* Query/key feature map phi (Alg. 1 step 3).  m = d for both. */
#define GRF_PHI_RELU      0     /* phi(x) = max(x, 0) elementwise: the map used in the paper's experiments */
#define GRF_PHI_IDENTITY  1     /* phi(x) = x: for tests */
#define GRF_PHI_ELU1      2     /* phi(x) = elu(x) + 1 (x + 1 for x > 0, exp(x) otherwise): the deterministic map of
                                   the linear transformer that Sec. 2 and Alg. 1 step 3 name as an alternative */

/* Message describing the last error returned on this thread.  Static storage; never free it. */
const char* grf_last_error(void);

/* Weighted adjacency matrix W of the graph G in CSR (Sec. 3.1).  Read-only.
 * Contract: row_ptr[0] = 0, row_ptr[n] = nnz, columns strictly ascending within a row, no self loops,
 * w finite.  deg(i) = row_ptr[i+1] - row_ptr[i] is the number of stored neighbours.  n, nnz < 2^31.
 * Every index read from row_ptr and col (here and in grf_phi) is range-checked on the device before it is used
 * as an address: an entry that breaks the contract ends the walk that meets it, respectively is skipped by the
 * attention calls, and the values that depend on it are unspecified. */
typedef struct grf_graph {
    int64_t        n;
    int64_t        nnz;
    const int32_t* row_ptr;   /* [n+1] */
    const int32_t* col;       /* [nnz] */
    const float*   w;         /* [nnz] */
} grf_graph;

/* GRF matrix Phi_hat (n x n, sparse) in CSR.  Row i is the feature phi_hat(v_i) of Eq. (GRF definition):
 * its stored columns are exactly the nodes visited by the walks out of v_i (ascending; a visited
 * node stays stored even if its summed value is 0; the diagonal is always present).
 * val holds n_f value planes that share row_ptr and col: plane h is at val + h * capacity. */
typedef struct grf_phi {
    int64_t  n;
    int64_t  capacity;        /* allocated entries of col and of each val plane */
    int32_t* row_ptr;         /* [n+1] */
    int32_t* col;             /* [capacity] */
    float*   val;             /* [n_f][capacity] */
} grf_phi;

/* ---------------------------------------------------------------------------------------------
 * Graph construction for dynamic point clouds (Sec. 4, point-cloud experiment; App. C): there the graph
 * changes at every step, walks cannot be precomputed, and the k-nearest-neighbour search is the stated
 * bottleneck.  The paper's solver is approximate and unspecified; this one is exact.
 *
 * points     device fp32 [n][3].
 * Neighbours of i: the k points j != i with the smallest squared distance, computed in fp32 as
 *            fl(fl(fl(dx*dx) + fl(dy*dy)) + fl(dz*dz)), dx = fl(x_i - x_j) (no fused multiply-add), ties going
 *            to the smaller index; fewer than k if n - 1 < k.  1 <= k <= 32.
 * symmetrise 0: row i holds its own k neighbours;  1: i ~ j if either lists the other.
 * weights    GRF_WEIGHT_INV_DEGREE: 1 / deg(i);  GRF_WEIGHT_EXP: exp(-dist / sigma);
 *            GRF_WEIGHT_GAUSS: exp(-dist^2 / (2 sigma^2));  the last two divided by their row sum (evaluated
 *            relative to the row's nearest neighbour, so a row far from everything is still finite).
 * Output     CSR as grf_graph expects it (columns ascending): row_ptr [n+1] always written; col, w [capacity]
 *            written when capacity >= nnz, else GRF_ECAPACITY with *nnz_out set.  grf_knn_graph_nnz_bound is
 *            always enough.  nnz_out is a HOST pointer; the call blocks on the stream once to fill it.  With
 *            nnz_out == NULL the call does not synchronise; capacity must then be at least the bound, the count
 *            stays on the device in row_ptr[n], and a grf_graph made from the result may carry nnz = capacity.
 * --------------------------------------------------------------------------------------------- */
#define GRF_WEIGHT_INV_DEGREE 0
#define GRF_WEIGHT_EXP        1
#define GRF_WEIGHT_GAUSS      2

int64_t grf_knn_graph_nnz_bound(int64_t n, int32_t k, int32_t symmetrise);     /* n*k or 2*n*k; -1 on bad arguments */
size_t grf_knn_graph_workspace_bytes(int64_t n, int32_t k);                    /* 0 on bad arguments */

grf_status grf_knn_graph(const float* points, int64_t n, int32_t k, int32_t symmetrise, int32_t weight_kind, float sigma,
                         void* workspace, size_t workspace_bytes, void* hip_stream,
                         int32_t* row_ptr, int32_t* col, float* w, int64_t capacity, int64_t* nnz_out);

/* ---------------------------------------------------------------------------------------------
 * Sampling (Alg. 1 steps 1-2; Sec. 3.3).
 *
 * From every node i, n_walks independent simple random walks are simulated.  Before every hop a walk
 * halts with probability p_halt, otherwise it moves to a uniformly chosen stored neighbour; it also
 * stops after f_len visited nodes (f vanishes beyond index f_len-1) or at a node without neighbours.
 * The prefix that reaches node q after t hops deposits
 *       f[t] * prod_{s<t} W[u_s,u_{s+1}] * deg(u_s) / (1 - p_halt)
 * into entry (i, q), and the row is divided by n_walks.
 *
 * Random stream (reproducible, independent of launch geometry): Philox4x32-10 with key
 * (seed & 0xffffffff, seed >> 32) and counter (node, walk, block, 0).  Block b serves hops 2b+1 and
 * 2b+2: words 0,1 are the (halt, neighbour) draws of hop 2b+1, words 2,3 those of hop 2b+2.
 * A walk halts iff halt_draw < floor(p_halt * 2^32) (evaluated in fp64 on the host); the neighbour is
 * entry floor(nbr_draw * deg / 2^32) of the CSR row.  Walk decisions are integer-only.
 * --------------------------------------------------------------------------------------------- */

/* Largest possible number of entries of Phi_hat: n * (1 + n_walks * (f_len - 1)).  -1 on bad arguments. */
int64_t grf_sample_nnz_bound(int64_t n, int32_t n_walks, int32_t f_len);

/* Bytes of workspace grf_sample needs (a multiple of 256).  0 on bad arguments. */
size_t grf_sample_workspace_bytes(int64_t n, int32_t n_walks, int32_t f_len, int32_t n_f);

/*
 * g            graph, device arrays.
 * f            HOST pointer, [n_f][f_len] row-major: n_f >= 1 modulation vectors that share one set of
 *              walks (Phi_hat is linear in f).  Copied before the call returns.
 * p_halt       in [0, 1].   n_walks >= 1.   f_len >= 1.
 * workspace    device, 256-byte aligned, >= grf_sample_workspace_bytes(...).
 * phi_out      caller-allocated.  row_ptr is always written.  col and the n_f planes of val are
 *              written when capacity >= nnz; otherwise GRF_ECAPACITY is returned (with *nnz_out set), so
 *              a first call with capacity 0 (col = val = NULL allowed) is a way to learn nnz.
 * nnz_out      HOST pointer; receives the number of entries.  The call blocks on the stream for this.
 *
 * Rows are assembled in LDS, by one wavefront per node (ranking by counting) or by a workgroup of 1024 threads per node
 * (a bitonic sorting network).  With cap = 1 + n_walks*(f_len-1), the largest possible number of deposits of a row: the
 * wavefront kernel serves cap <= 768, the workgroup kernel cap > 8192, and in between the one that a cost model in n,
 * n_walks, f_len and p_halt (the expected deposits and hops) says is faster.  The pattern does not depend on the
 * choice; values differ by the order of their sums.
 * GRF_EUNSUPPORTED if 1 + n_walks*(f_len-1) exceeds 16384 or if the number of entries does not fit int32.
 */
grf_status grf_sample(const grf_graph* g,
                      const float* f, int32_t f_len, int32_t n_f,
                      double p_halt, int32_t n_walks, uint64_t seed,
                      void* workspace, size_t workspace_bytes, void* hip_stream,
                      grf_phi* phi_out, int64_t* nnz_out);

/* The same sampling as stream-ordered work only, for callers that must not touch the host (HIP graph capture,
 * tight loops): f_device is a DEVICE pointer [n_f][f_len] read when the kernels run (so a training loop can update
 * it in place), nothing is synchronised and no count comes back: phi_out->capacity must be at least
 * grf_sample_nnz_bound() and the number of entries stays on the device in phi_out->row_ptr[n].  The attention
 * calls accept phi_out with nnz = capacity (see there).  Workspace as for grf_sample. */
grf_status grf_sample_async(const grf_graph* g,
                            const float* f_device, int32_t f_len, int32_t n_f,
                            double p_halt, int32_t n_walks, uint64_t seed,
                            void* workspace, size_t workspace_bytes, void* hip_stream,
                            grf_phi* phi_out);

/* The walks alone, for inspection: traj is device [n][n_walks][max_nodes] int32; entry t of a walk is
 * the node visited after t hops, or -1 past its end.  Same stream as grf_sample with f_len = max_nodes. */
grf_status grf_sample_walks(const grf_graph* g, double p_halt, int32_t n_walks, int32_t max_nodes,
                            uint64_t seed, void* hip_stream, int32_t* traj);

/* ---------------------------------------------------------------------------------------------
 * Masked linear attention (Eq. 7; Alg. 1 steps 3-5), evaluated without ever forming the N x Nm
 * matrices Phi_{Q,G}, Phi_{K,G}:
 *
 *   buckets   S_l = sum_j Phi_hat[j,l] phi(k_j) v_j^T  (d x d),  z_l = sum_j Phi_hat[j,l] phi(k_j)  (d)
 *             -- block l of Phi_{K,G}^T V and of Phi_{K,G}^T 1
 *   gather    num_i = sum_l Phi_hat[i,l] phi(q_i)^T S_l,   den_i = sum_l Phi_hat[i,l] phi(q_i)^T z_l
 *             out_i = num_i / den_i      (no epsilon: den_i = 0 gives IEEE inf/NaN, not an error)
 *
 * Cost is linear in nnz(Phi_hat) except for the ordering of the column lists, which is quadratic in the length of a
 * column (spread over the whole device); a bucket is summed by one wavefront, so a single column with very many
 * entries (a hub node) is correct but serial in that part.
 *
 * Q, K, V    contiguous [B][H][n][d], dtype GRF_DTYPE_F32 or GRF_DTYPE_BF16.  d in {32, 64}.
 * phi, nnz   Phi_hat and its number of entries.  nnz may also be any upper bound on phi->row_ptr[n] up to
 *            phi->capacity (the kernels take the end of the rows from row_ptr[n]; nnz sizes the workspace and the
 *            strides in it), which is what a caller has who sampled without waiting for the count (see grf_sample).
 *            n_f value planes: n_f == 1 is shared
 *            by all heads, n_f == H gives head h plane h.  One graph per call, shared over the batch.
 * --------------------------------------------------------------------------------------------- */

/* Floats per bucket record: d*d of S_l (feature index major: S_l[a][c] at a*d + c) followed by d of z_l. */
int64_t grf_bucket_record_floats(int32_t d);

/* Workspace bytes of grf_masked_linear_attention (multiple of 256; 0 on bad arguments): the column
 * lists of Phi_hat plus the bucket records of bh_chunk slices.
 * bh_chunk: how many (batch, head) slices have their buckets resident at once; <= 0 means all B*H. */
size_t grf_attention_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk);

/* Workspace bytes of grf_form_buckets (the column lists of Phi_hat only, with n_f value planes). */
size_t grf_buckets_workspace_bytes(int64_t n, int64_t nnz, int32_t n_f);

/* Buckets only (Alg. 1 step 5, the two Phi_{K,G}^T products).
 * buckets: device [B*H][n][grf_bucket_record_floats(d)] fp32, fully overwritten. */
grf_status grf_form_buckets(const void* K, const void* V, int32_t dtype,
                            int64_t B, int64_t H, int64_t n, int32_t d,
                            const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                            void* workspace, size_t workspace_bytes, void* hip_stream,
                            float* buckets);

/* Gather only (Alg. 1 step 5, the Phi_{Q,G} products and D^-1), from records laid out as
 * grf_form_buckets writes them.  Needs no workspace.  Outputs as below. */
grf_status grf_gather_buckets(const void* Q, int32_t dtype,
                              int64_t B, int64_t H, int64_t n, int32_t d,
                              const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                              const float* buckets, void* hip_stream,
                              float* out, float* num_opt, float* den_opt);

/* The whole attention call: column lists, then buckets and gather per chunk of slices.
 * out       device [B][H][n][d] fp32.
 * num_opt   device [B][H][n][d] fp32 or NULL;  den_opt  device [B][H][n] fp32 or NULL. */
grf_status grf_masked_linear_attention(const void* Q, const void* K, const void* V, int32_t dtype,
                                       int64_t B, int64_t H, int64_t n, int32_t d,
                                       const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                       int32_t bh_chunk,
                                       void* workspace, size_t workspace_bytes, void* hip_stream,
                                       float* out, float* num_opt, float* den_opt);

/* ---------------------------------------------------------------------------------------------
 * Bucket-fused variant of the whole attention call: same inputs, outputs and error behaviour as
 * grf_masked_linear_attention, same num, den, out up to fp32 summation order, but S_l is never
 * written to memory.  It rests on Eq. 6: queries and keys share the graph features, so the rows that
 * consume bucket l are the rows that contribute to it; per bucket the kernel forms S_l and z_l in
 * registers, multiplies them at once by the weighted phi(q) of the same rows, and streams out one
 * d-float partial numerator and one partial denominator per entry of Phi_hat; a second kernel sums
 * each row's partials in ascending-l order (deterministic; no float atomics).
 * At d = 64 the two contractions run on the bf16 matrix instructions with fp32 accumulation.  fp32 operands
 * enter as the sum of three bf16 numbers (exact: 3 x 8 significant bits) and a product is formed from the six
 * piece products that matter (what is dropped is at most 2^-23 of the product): fp32 accuracy.  With bf16 inputs and a feature map that keeps bf16 values bf16
 * (ReLU, identity) the operand that is not a bf16 number as stored (Phi_hat[j,l] phi(k_j), then S_l) enters as
 * the sum of two bf16 numbers, a relative error of at most 2^-16 on that operand.  d = 32 uses the fp32 matrix
 * instructions.  Which of these runs depends on d, dtype and feature_map only.  Range: a bf16 number has the exponent
 * range of an fp32 number, so nothing overflows that would not in fp32, except magnitudes within one part in 256
 * of the largest finite fp32 number, whose leading piece rounds to infinity.  At the small end the third piece of an
 * operand x carries bits down to 2^-23 |x| and bf16 (subnormals included, which the conversions and the matrix
 * instructions honour) reaches down to 2^-133: operands of magnitude 2^-110 and more are split exactly, smaller ones
 * lose low bits gradually (a relative error of up to 2^-8 on an operand at 2^-126).  Measured: scaling Q, K, V or
 * Phi_hat by powers of two between 2^-95 and 2^100 changes no mantissa bit of num and den.
 * At d = 64 lists of at most 32 entries are not evaluated through S_l at all but through the entry-by-entry dot
 * products of their rows, several buckets per wavefront (cheaper below d entries per list); same products, same bars.
 * Workspace: column lists plus (d + 1) floats per entry of Phi_hat per resident slice. */
size_t grf_fused_attention_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk);

grf_status grf_masked_linear_attention_fused(const void* Q, const void* K, const void* V, int32_t dtype,
                                             int64_t B, int64_t H, int64_t n, int32_t d,
                                             const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                             int32_t bh_chunk,
                                             void* workspace, size_t workspace_bytes, void* hip_stream,
                                             float* out, float* num_opt, float* den_opt);

/* ---------------------------------------------------------------------------------------------
 * Prepared column lists.  For a fixed graph the walks are sampled once and frozen for each attention head and layer
 * (Sec. 4, image experiments), so the column lists of Phi_hat, which grf_form_buckets, the whole attention calls and
 * the backward call otherwise rebuild on every call, can be built once:
 *
 *   grf_phi_prepare          writes the column lists of phi (with its n_f value planes in list order and the launch
 *                            plans of the bucket kernels) into `prepared`, a caller-owned device buffer of
 *                            grf_phi_prepare_bytes(n, nnz, n_f) bytes, 256-byte aligned.  Stream-ordered, no
 *                            synchronisation.  The buffer stays valid while phi's pattern (row_ptr, col) is unchanged.
 *   grf_phi_prepare_values   refreshes only the value planes inside `prepared` from phi->val: for a modulation f that
 *                            has changed (training) over the same walks.
 *   *_prepared               the attention calls with `prepared` in place of the rebuild: same arguments, results
 *                            bit-identical to the call without the suffix.  n, nnz and n_f must be the values given to
 *                            grf_phi_prepare (they fix the layout of the buffer).  Workspace: that of the call without
 *                            the suffix minus grf_phi_prepare_bytes(n, nnz, n_f) (grf_form_buckets_prepared: none).
 * The contents of `prepared` are trusted like a pointer argument: a buffer that grf_phi_prepare did not fill for
 * this phi, nnz and n_f is undefined behaviour.
 * --------------------------------------------------------------------------------------------- */
size_t grf_phi_prepare_bytes(int64_t n, int64_t nnz, int32_t n_f);      /* 0 on bad arguments */

grf_status grf_phi_prepare(const grf_phi* phi, int64_t nnz, int32_t n_f, void* prepared, size_t prepared_bytes, void* hip_stream);

grf_status grf_phi_prepare_values(const grf_phi* phi, int64_t nnz, int32_t n_f, void* prepared, size_t prepared_bytes, void* hip_stream);

grf_status grf_form_buckets_prepared(const void* K, const void* V, int32_t dtype,
                                     int64_t B, int64_t H, int64_t n, int32_t d,
                                     const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                     const void* prepared, size_t prepared_bytes, void* hip_stream, float* buckets);

grf_status grf_masked_linear_attention_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
                                                int64_t B, int64_t H, int64_t n, int32_t d,
                                                const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                int32_t bh_chunk, const void* prepared, size_t prepared_bytes,
                                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                                float* out, float* num_opt, float* den_opt);

grf_status grf_masked_linear_attention_fused_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
                                                      int64_t B, int64_t H, int64_t n, int32_t d,
                                                      const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                      int32_t bh_chunk, const void* prepared, size_t prepared_bytes,
                                                      void* workspace, size_t workspace_bytes, void* hip_stream,
                                                      float* out, float* num_opt, float* den_opt);

/* grf_masked_linear_attention_fused for callers that can neither allocate device memory nor hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Inputs, outputs,
 * results (bit-identical to grf_masked_linear_attention_fused) and error behaviour are the same; the scratch
 * memory (column lists of Phi_hat, partial rows) is a 64 MiB device array that is part of the loaded library, one
 * copy per GPU, held until the process ends.  The call allocates nothing, frees nothing and does not synchronise;
 * it splits the B*H slices into as many chunks as the array requires.
 * Limit: grf_fused_attention_workspace_bytes(B, H, n, d, nnz, n_f, 1) <= 64 MiB (about 230 000 entries of Phi_hat
 * at d = 64 and n_f = 1), else GRF_EUNSUPPORTED and nothing is launched.
 * Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (different streams,
 * different host threads) race on it and must be ordered by the caller. */
grf_status grf_masked_linear_attention_fused_static(const void* Q, const void* K, const void* V, int32_t dtype,
                                                    int64_t B, int64_t H, int64_t n, int32_t d,
                                                    const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                    void* hip_stream, float* out, float* num_opt, float* den_opt);

/* ---------------------------------------------------------------------------------------------
 * Asymmetric graph random features (App. D, Alg. 2): the keys use the one-hot feature (f^(2) = delta_0,
 * Phi^(2) = I), so the mask estimate is the sampled matrix itself.  phi must have been sampled with
 * f = alpha (the mask's own Taylor coefficients), and
 *     num_i = sum_j Phi_hat[i,j] (phi(q_i) . phi(k_j)) v_j,    den_i = sum_j Phi_hat[i,j] (phi(q_i) . phi(k_j)),
 *     out_i = num_i / den_i
 * (the appendix's per-walk accumulation, with a row's deposits already summed per end node; the
 * factor n in its printed normalisation has no counterpart in the accumulations and is not applied).
 * Arguments, layouts, n_f and error behaviour as for grf_masked_linear_attention; needs no workspace. */
grf_status grf_asymmetric_masked_attention(const void* Q, const void* K, const void* V, int32_t dtype,
                                           int64_t B, int64_t H, int64_t n, int32_t d,
                                           const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                           void* hip_stream, float* out, float* num_opt, float* den_opt);

/* ---------------------------------------------------------------------------------------------
 * Gradients, for training with the learnable modulation f of Alg. 1 (and through Q, K, V).
 *
 * The forward pass is out = attention(Q, K, V, Phi_hat) with Phi_hat = sample(f), linear in f.  Given
 * d_out = dL/dout, grf_masked_linear_attention_backward returns dL/dQ, dL/dK, dL/dV and dL/dPhi_hat on the
 * stored entries; grf_sample_backward then contracts dL/dPhi_hat with the per-hop walk loads to give dL/df.
 *
 * With v'_j = [v_j, 1] and g'_i = [d_out_i / den_i, -(d_out_i . out_i) / den_i] (chain rule through the division
 * of Eq. 7), S'_l = sum_j Phi[j,l] phi(k_j) v'_j^T and T'_l = sum_i Phi[i,l] phi(q_i) g'_i^T,
 *     dL/dphi(q_i) = sum_l Phi[i,l] S'_l g'_i          dL/dphi(k_j) = sum_l Phi[j,l] T'_l v'_j
 *     dL/dv_j      = sum_l Phi[j,l] T_l^T phi(k_j)     dL/dPhi[i,l] = phi(q_i)^T S'_l g'_i + phi(k_i)^T T'_l v'_i
 * and dL/dq = dL/dphi(q) * phi'(q) elementwise, likewise k.  Evaluated bucket by bucket like the fused forward
 * pass (the rows that consume bucket l are its contributors), in three passes of two MFMA contractions each;
 * per-entry partial rows are summed per output row in ascending-l order (deterministic, no float atomics).
 * At d = 64 the contractions run on the bf16 matrix instructions with fp32 accumulation, operands entering as
 * sums of bf16 numbers: three pieces and six piece products per product with fp32 inputs (fp32 accuracy), two
 * pieces and three piece products with bf16 inputs (relative error at most 2^-16 per operand).
 *
 * Q, K, V, dtype, B, H, n, d, phi, nnz, n_f, feature_map, bh_chunk: as in the forward call.
 * out, den   device fp32 [B][H][n][d] and [B][H][n]: the forward results (out and den_opt of either variant).
 * d_out      device fp32 [B][H][n][d].
 * dQ, dK, dV device fp32 [B][H][n][d], overwritten.
 * dphi_val   device fp32 [n_f][phi->capacity] or NULL: plane h receives the sum over the (batch, head) slices
 *            that use plane h of dL/dPhi_hat.  When nnz is an upper bound, the entries between the end of the rows
 *            (phi->row_ptr[n]) and nnz receive 0; entries [nnz, capacity) are not touched.
 * A row with den_i = 0 propagates IEEE inf/NaN into every gradient it touches (no epsilon, as in the forward).
 * --------------------------------------------------------------------------------------------- */
size_t grf_attention_backward_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk);

grf_status grf_masked_linear_attention_backward(const void* Q, const void* K, const void* V, int32_t dtype,
                                                int64_t B, int64_t H, int64_t n, int32_t d,
                                                const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                const float* out, const float* den, const float* d_out,
                                                int32_t bh_chunk,
                                                void* workspace, size_t workspace_bytes, void* hip_stream,
                                                float* dQ, float* dK, float* dV, float* dphi_val);

/* The same over prepared column lists (see grf_phi_prepare). */
grf_status grf_masked_linear_attention_backward_prepared(const void* Q, const void* K, const void* V, int32_t dtype,
                                                         int64_t B, int64_t H, int64_t n, int32_t d,
                                                         const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                         const float* out, const float* den, const float* d_out,
                                                         int32_t bh_chunk, const void* prepared, size_t prepared_bytes,
                                                         void* workspace, size_t workspace_bytes, void* hip_stream,
                                                         float* dQ, float* dK, float* dV, float* dphi_val);

/* Backward of grf_asymmetric_masked_attention (App. D): with a_ij = phi(q_i).phi(k_j) and c_ij = v'_j . g'_i,
 *     dL/dPhi[i,j] = a_ij c_ij                      dL/dphi(q_i) = sum_j Phi[i,j] c_ij phi(k_j)
 *     dL/dphi(k_j) = sum_i Phi[i,j] c_ij phi(q_i)   dL/dv_j      = sum_i Phi[i,j] a_ij g_i
 * (row sums in one kernel, column sums over the column lists in a second; fixed summation order).
 * Arguments as for grf_masked_linear_attention_backward; dL/df follows from grf_sample_backward as before,
 * since Phi_hat is the same sampled matrix (with f = alpha). */
size_t grf_asymmetric_backward_workspace_bytes(int64_t B, int64_t H, int64_t n, int32_t d, int64_t nnz, int32_t n_f, int32_t bh_chunk);

grf_status grf_asymmetric_masked_attention_backward(const void* Q, const void* K, const void* V, int32_t dtype,
                                                    int64_t B, int64_t H, int64_t n, int32_t d,
                                                    const grf_phi* phi, int64_t nnz, int32_t n_f, int32_t feature_map,
                                                    const float* out, const float* den, const float* d_out,
                                                    int32_t bh_chunk,
                                                    void* workspace, size_t workspace_bytes, void* hip_stream,
                                                    float* dQ, float* dK, float* dV, float* dphi_val);

/* Gradient of the sampled features with respect to the modulation (Eq. GRF definition is linear in f):
 *     df[h][t] = (1 / n_walks) * sum over nodes i, walks k with at least t hops of
 *                load_{k,t} * dphi_val[h][entry (i, node visited by walk k after t hops)]
 * over the same walks as grf_sample with the same (g, p_halt, n_walks, seed, f_len).
 * phi        the pattern sampled with those arguments (row_ptr, col; val is not read), nnz its entries.
 * dphi_val   device fp32 [n_f][phi->capacity].
 * df         device fp32 [n_f][f_len], overwritten.  Sums run in a fixed order (bitwise reproducible).
 * Workspace: n * n_f * f_len floats of per-node partial sums (plus staging areas when rows are assembled by workgroups). */
size_t grf_sample_backward_workspace_bytes(int64_t n, int32_t n_walks, int32_t f_len, int32_t n_f);

grf_status grf_sample_backward(const grf_graph* g, int32_t f_len, int32_t n_f,
                               double p_halt, int32_t n_walks, uint64_t seed,
                               const grf_phi* phi, int64_t nnz, const float* dphi_val,
                               void* workspace, size_t workspace_bytes, void* hip_stream,
                               float* df);

/* Testing aid, not part of the method.  The bucket kernels (grf_form_buckets, the fused call, the backward call)
 * address rows of Q, K, V with 32-bit byte offsets when a [n][d] fp32 slice is below 4 GiB and with 64-bit offsets
 * otherwise; on != 0 makes every later call in this process take the 64-bit form, so that it can be tested at small
 * sizes.  Results are the same bits either way. */
void grf_debug_force_wide_offsets(int32_t on);

/* Testing and tuning aid, not part of the method.  grf_sample, grf_sample_async and grf_sample_backward assemble the
 * rows of a node with one of two kernels (one wavefront per node, ranking by counting; one workgroup per node, sorting
 * network), chosen by a cost model from n, n_walks, f_len and p_halt wherever both can serve, that is between 769 and
 * 8192 possible deposits per node.  which = 1 / 2 makes every later call in this process take the wavefront / the
 * workgroup kernel in that range, 0 restores the choice.  Pattern and row_ptr are the same bits either way; values
 * differ by the order of their sums (the workgroup kernel adds in (walk, hop) order).  which = 3 is 1 with the
 * wavefront kernel ordering deposits by (column, slot) as two words instead of one packed 32-bit key, the form it
 * otherwise takes only when n * 2^ceil(log2(cap)) exceeds 2^32; same bits as which = 1. */
void grf_debug_force_row_kernel(int32_t which);

#ifdef __cplusplus
}
#endif
#endif /* GRF_H_ */
