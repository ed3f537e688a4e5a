/*
 * gcn.h -- C ABI of the single-GPU hot path of full-batch GCN training on MI355X (gfx950).
 *
 * The operations are those of "Reducing Communication in Graph Neural Network Training"
 * (arXiv 2005.03300): per layer Z^l = A^T H^{l-1} W^l, H^l = sigma(Z^l) ("Forward Propagation"),
 * and the three backward equations of "Backpropagation Derivations".  This library is what one
 * process of the paper's 1D algorithm runs between its collectives, on the whole graph.
 *
 * Conventions for every call
 *   - Every pointer named "device" is HIP device memory on the current device; "host" is host
 *     memory.  Dense matrices are fp32, row-major, with a leading dimension in elements.
 *   - Dense buffers are owned by the caller; the library neither frees nor keeps them after the
 *     work queued on `stream` has finished.  Only gcn_csr objects own device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute calls only
 *     queue work on it and return; gcn_csr_create*, gcn_csr_info, gcn_csr_destroy and the prepare calls
 *     synchronise.  A sparse product whose width was not prepared (gcn_spmm_prepare, gcn_epoch_prepare) and
 *     was not used before may build and keep another stored order of the matrix and grow the handle's
 *     buffers: it then allocates device memory and waits for the stream once.  After a prepare call for the
 *     widths in use, the products and the epoch calls only queue kernels and device-to-device copies: they
 *     can be captured in a HIP graph from their first call on.  Nothing the library has handed to a kernel is
 *     freed before gcn_csr_destroy (a larger buffer replaces a smaller one, which is kept), so graphs captured
 *     earlier stay valid.
 *   - Library-owned scratch exists only for the stand-alone gcn_gemm (ta = 1), gcn_softmax_nll* and the bias
 *     gradient of gcn_layer_backward: one buffer per (device, stream), grown on demand by the first call that
 *     needs more (an allocation), never shared between streams; gcn_scratch_release frees all of them.  The
 *     epoch calls keep these partial sums in the caller's workspace instead.
 *   - Every function returns GCN_OK (0) or a negative GCN_ERR_* code and never throws or aborts.
 *     gcn_last_error() returns a thread-local message for the last failure on this thread.
 *   - No call is safe to run concurrently with another call that uses the same gcn_csr.  Calls on different
 *     matrices, or calls without a matrix on different streams, may run concurrently from different threads.
 */
#ifndef GCN_H
#define GCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GCN_OK 0
#define GCN_ERR_BADARG (-1)      /* NULL pointer, non-positive size, ld < width, aliasing */
#define GCN_ERR_RANGE (-2)       /* vertex id outside [0,n), n >= 2^31, counts that overflow */
#define GCN_ERR_NOTRANSPOSE (-3) /* trans=1 asked of a matrix built without GCN_BUILD_TRANSPOSE */
#define GCN_ERR_OOM (-4)         /* device allocation failed */
#define GCN_ERR_WORKSPACE (-5)   /* caller workspace too small */
#define GCN_ERR_HIP (-6)         /* a HIP runtime call failed; see gcn_last_error() */
#define GCN_ERR_UNSORTED (-7)    /* caller-supplied CSR has unsorted/duplicate/out-of-range columns */

/* gcn_csr_create flags */
#define GCN_SYMMETRISE 1u      /* store (v,u) for every input (u,v) */
#define GCN_ADD_SELF_LOOPS 2u  /* insert exactly one diagonal entry per row */
#define GCN_NORM_SYM 4u        /* values 1/sqrt(d_i d_j); without it every value is 1.0f */
#define GCN_BUILD_TRANSPOSE 8u /* also store A^T in compressed rows (needed for trans=1) */
#define GCN_NORM_ROW 16u       /* values 1/d_i (row normalisation D^-1 (A+I), for directed graphs); not with NORM_SYM */

/* gcn_spmm / gcn_gemm epilogues */
#define GCN_EPI_NONE 0
#define GCN_EPI_RELU 1 /* out = max(out, 0) */
#define GCN_EPI_MASK 2 /* out = Zprev > 0 ? out : 0   (Hadamard product with sigma'(Zprev)) */

/* association order of A^T H W */
#define GCN_ORDER_AUTO 0       /* GEMM first if f_out <= f_in, else SpMM first */
#define GCN_ORDER_GEMM_FIRST 1 /* A^T (H W) */
#define GCN_ORDER_SPMM_FIRST 2 /* (A^T H) W  -- the order of the paper's Algorithm 1 */

#define GCN_ACT_NONE 0
#define GCN_ACT_RELU 1

/* gcn_config / gcn_csr_config keys */
#define GCN_CFG_SPMM_ALGO 1 /* 0 = automatic, 1 = one thread per output element, 2 = nonzero-split, 3 = column sweep, 4 = hub schedule (long rows x hot columns over a packed buffer, the rest as 2) */
#define GCN_CFG_TIMING 2    /* 1 = bracket the dominant kernels with HIP events (see gcn_timing_read) */
#define GCN_CFG_SPMM_BLOCKS 3 /* column blocks of the SpMM: 0 = automatic, 1 = never block, k >= 2 = k blocks */
#define GCN_CFG_SWEEP_HEAVY 4 /* rows longer than this bypass the column sweep (default 1024; >= 1) */
#define GCN_CFG_SWEEP_WAVES 5 /* column sweep: tasks per compute unit in one launch (default 9: 9 x 16 KB of LDS accumulators per compute unit, the most that fit; 1..18) */
#define GCN_CFG_PATTERN_SPMM 6 /* gcn_spmm and gcn_epoch* on a matrix made by gcn_csr_create with GCN_NORM_SYM: use the value-free SpMM (operand rows pre-scaled by d^-1/2, output rows scaled by d^-1/2) instead of reading the stored values. 0 never, 1 always, 2 (default) when the mean row has at least 64 entries */
#define GCN_CFG_HUB_MB 7   /* hub schedule: size in MB of the packed buffer that holds the rows of X selected by the columns with the most entries (default 32) */
#define GCN_CFG_HUB_DMIN 8 /* hub schedule: rows with at least this many entries are treated as long rows (default 64) */
#define GCN_CFG_HUB_BLOCK_COLS 9 /* hub schedule: columns per block of the packed buffer (0, default: about 2 MB of the gathered panel; a multiple of 64) */
#define GCN_CFG_SPLIT_LDS_KB 10 /* nonzero-split kernel for operands of up to 16 floats: LDS per workgroup in KB, padding included (18..64, default 28; 18 = no padding).  Padding lowers the number of resident wavefronts, which keep 64 gathers in flight each */

#define GCN_CFG_FUSED_LAST_LAYER 11 /* gcn_epoch*: when the last layer runs SpMM-first at f_in = 16 with at most 256 classes, one kernel per 16-row strip of A^T H computes the logits, the loss, G^L, the weight gradient and G^L W^T, and the n x C matrices Z^L and G^L are not written to memory.  1 (default): fused, gcn_epoch_view of the last layer then points at memory the epoch did not write; 2: fused and Z^L, G^L stored for inspection; 0: separate kernels (stored) */

typedef struct gcn_csr gcn_csr; /* opaque: A (and A^T) in compressed rows, degrees, schedules */

/* -------------------------------------------------------------------------------------------
 * Graph construction -- section "Graph Neural Networks": the adjacency matrix with added
 * self-connections, scaled to D^-1/2 (A+I) D^-1/2 with D the modified degrees; section
 * "Communication Schemes and their Analyses": both A and A^T are stored.
 *
 * src, dst: DEVICE int32[n_edges], borrowed for the call.  Pairs with src == dst are dropped,
 * duplicates collapse to one entry.  The result has columns ascending in every row; rowptr is
 * int64, colidx int32, val fp32, deg int32 = entries per row of A.  With GCN_NORM_SYM,
 * val(i,j) = (float)(1.0 / sqrt((double)deg_i * (double)deg_j)); with GCN_NORM_ROW, (float)(1.0 / (double)deg_i).
 * The rows of a graph without self loops can be empty; with GCN_NORM_SYM an entry that touches a vertex whose
 * row is empty gets the value 0 (D^-1/2 as a pseudo-inverse), and gcn_csr_inv_sqrt_degrees gives 0 for it.
 * Errors: BADARG (NULL out, n <= 0, n_edges < 0, NULL arrays with n_edges > 0), RANGE (n >= 2^31
 * or an id outside [0,n)), OOM, HIP.  On error *out is NULL.
 * ----------------------------------------------------------------------------------------- */
int gcn_csr_create(gcn_csr** out, int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                   uint32_t flags, void* stream);

/* Adopt a caller-built compressed-row matrix (DEVICE arrays, copied).  val == NULL means 1.0f.
 * Columns must be strictly ascending per row and inside [0,n): otherwise UNSORTED.  Rows may be
 * empty.  flags: only GCN_BUILD_TRANSPOSE is honoured. */
int gcn_csr_create_from_csr(gcn_csr** out, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                            const float* val, uint32_t flags, void* stream);

/* The same for a rectangular n_rows x n_cols matrix -- one process's block row of the paper's 1D
 * algorithm ("A One-Dimensional (1D) Algorithm": rows [i n/P, (i+1) n/P) of A^T against all of H).
 * gcn_spmm with trans=0 reads X with n_cols rows and writes Z with n_rows rows; trans=1 the other way
 * round.  The layer and epoch calls need a square matrix. */
int gcn_csr_create_from_csr_rect(gcn_csr** out, int64_t n_rows, int64_t n_cols, const int64_t* rowptr,
                                 const int32_t* colidx, const float* val, uint32_t flags, void* stream);

int gcn_csr_destroy(gcn_csr* a);

/* Sizes; any output pointer may be NULL. */
int gcn_csr_info(const gcn_csr* a, int64_t* n, int64_t* nnz, int32_t* max_degree);

/* Rows and columns of A (equal unless made by gcn_csr_create_from_csr_rect). */
int gcn_csr_shape(const gcn_csr* a, int64_t* n_rows, int64_t* n_cols);

/* DEVICE pointers to the stored arrays (valid until destroy) for bit-exact checks.
 * transposed=1 selects A^T (NOTRANSPOSE if absent); deg is always that of A. */
int gcn_csr_arrays(const gcn_csr* a, int transposed, const int64_t** rowptr, const int32_t** colidx,
                   const float** val, const int32_t** deg);

/* Copy the stored arrays into caller-owned DEVICE buffers (rowptr int64[n+1], colidx int32[nnz],
 * val float[nnz], deg int32[n]); any destination may be NULL.  Queued on `stream`. */
int gcn_csr_export(const gcn_csr* a, int transposed, int64_t* rowptr, int32_t* colidx, float* val, int32_t* deg,
                   void* stream);

/* -------------------------------------------------------------------------------------------
 * SpMM -- the local sparse-dense product of sections "Graph Neural Networks" and "A
 * One-Dimensional (1D) Algorithm":  Z[i,:] = sum over stored entries k of row i of op(A) of
 * val[k] * X[col[k],:], op(A) = A (trans=0) or A^T (trans=1).
 * X: device n x f, ld ldx >= f.  Z: device n x f, ld ldz >= f, must not overlap X (for a rectangular
 * matrix X has as many rows as op(A) has columns and Z as many as op(A) has rows).
 * epilogue GCN_EPI_MASK reads Zprev (device n x f, ld ldzprev); otherwise Zprev is ignored.
 * Sums are fp32 and run-to-run reproducible (no floating-point atomics).  The first call at a
 * given width may build and cache a column-blocked copy of the matrix inside `a` (it allocates
 * and synchronises once); later calls only queue kernels.
 * For a matrix that gcn_csr_create normalised symmetrically the same product is D^-1/2 ((A+I) (D^-1/2 X)); when
 * GCN_CFG_PATTERN_SPMM says so (by default: mean row of at least 64 entries) it is computed in that form, without
 * reading the stored values: X is copied with its rows scaled into a buffer of the handle (n x f floats, allocated by
 * gcn_spmm_prepare or by the first call at that width), the gathered rows are summed and the output rows scaled.  The
 * result differs from the sum over val[k] by fp32 roundings only (a few 1e-7 of the result's rms).
 * ----------------------------------------------------------------------------------------- */
int gcn_spmm(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
             int epilogue, const float* Zprev, int64_t ldzprev, void* stream);

/* Builds, for operands of width f (16-byte aligned, leading dimensions multiples of 4 when f is), whatever
 * gcn_spmm / gcn_spmm_pattern would build or grow on their first call at that width -- the stored order the
 * schedule needs and the handle's buffers -- without running a product.  Synchronises `stream`.  Copies for
 * several widths are kept side by side, so a model whose products alternate between widths never rebuilds.
 * gcn_spmm_describe writes the schedule such a product takes and its launch shape as text into `out`
 * (host, out_bytes including the terminator; truncated if too small), building it like gcn_spmm_prepare if
 * needed; reports and tests use it to tie a measurement to the schedule it was taken on. */
int gcn_spmm_prepare(gcn_csr* a, int trans, int32_t f, void* stream);
int gcn_spmm_describe(gcn_csr* a, int trans, int32_t f, char* out, size_t out_bytes, void* stream);

/* -------------------------------------------------------------------------------------------
 * gcn_spmm for callers that cannot allocate device memory: code under HIP graph capture from its
 * first call on, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, result and
 * errors as gcn_spmm, always through the nonzero-split kernel over the stored order (so the result is
 * bit-identical to gcn_spmm with GCN_CFG_SPMM_ALGO = 2 and GCN_CFG_SPMM_BLOCKS = 1), but the partial rows of
 * rows that cross wavefronts (f floats per 512 stored entries) live in a fixed array of
 * GCN_SPMM_STATIC_SCRATCH_BYTES inside the library's device image instead of a buffer the handle grows.
 * The call makes no hipMalloc / hipFree and no allocating library call; it only queues kernels on `stream`.
 * GCN_ERR_WORKSPACE when ceil(nnz / 512) * f * 4 bytes exceed the array (e.g. more than 134 M stored entries
 * at f = 16); BADARG when the matrix lives on another device than the current one.
 * Every call on a GPU shares that GPU's array (each GPU holds its own copy until the process ends): calls that
 * overlap in time on one GPU (different streams or threads) race on it.  Nothing in it has to start at
 * zero -- every partial row is written by the product before it is read -- so consecutive calls need no clearing.
 * ----------------------------------------------------------------------------------------- */
#define GCN_SPMM_STATIC_SCRATCH_BYTES (16u << 20)
int gcn_spmm_static(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                    int epilogue, const float* Zprev, int64_t ldzprev, void* stream);

/* -------------------------------------------------------------------------------------------
 * Value-free SpMM for the symmetric normalisation of section "Graph Neural Networks":
 * D^-1/2 (A+I) D^-1/2 X = D^-1/2 ((A+I) (D^-1/2 X)), so the stored values need not be read.
 *   gcn_spmm_pattern:  Z[i,:] = epilogue(row_scale[i] * sum over stored entries k of row i of
 *                      op(A) of X[col[k],:]);  the stored values are ignored; row_scale (device,
 *                      one float per row of op(A)) may be NULL (= 1).  Other arguments, layout,
 *                      reproducibility and errors as gcn_spmm.
 *   gcn_scale_rows:    Y[i,:] = scale[i] * X[i,:]  (rows x cols, device; Y may be X).
 *   gcn_csr_inv_sqrt_degrees:  out[i] = (float)(1/sqrt((double)d_i)) with d the stored entries per
 *                      row of A (device, n floats; BADARG for a rectangular matrix).
 * With s = inv_sqrt_degrees, gcn_scale_rows(X, s) followed by gcn_spmm_pattern(row_scale = s)
 * equals gcn_spmm on a GCN_NORM_SYM matrix up to fp32 rounding (about 2^-23 relative per term).
 * ----------------------------------------------------------------------------------------- */
int gcn_spmm_pattern(gcn_csr* a, int trans, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                     const float* row_scale, int epilogue, const float* Zprev, int64_t ldzprev, void* stream);
int gcn_scale_rows(int64_t rows, int32_t cols, const float* X, int64_t ldx, const float* scale, float* Y, int64_t ldy,
                   void* stream);
int gcn_csr_inv_sqrt_degrees(const gcn_csr* a, float* out, void* stream);

/* -------------------------------------------------------------------------------------------
 * Dense products of "Forward Propagation" (H W) and of Equations 2 and 3 (S W^T, H^T S):
 * C = op(A) op(B) [+ 1 bias^T], then the epilogue.  op(A) is M x K, op(B) is K x N; ta/tb != 0
 * mean the stored matrix is the transpose (stored A is K x M, stored B is N x K).  All device,
 * row-major.  bias (N floats) may be NULL.  ta=1 sums over the long dimension K in a fixed
 * order (reproducible); it uses a library-owned scratch buffer.  ta=1 with tb=1 is BADARG.
 * ----------------------------------------------------------------------------------------- */
int gcn_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
             const float* B, int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue,
             const float* Zprev, int64_t ldzprev, void* stream);

/* sigma and sigma' of "Forward Propagation" / Equations 1-2 as stand-alone element-wise calls
 * over rows x cols matrices with leading dimensions. out may equal the first input. */
int gcn_relu(int64_t rows, int32_t cols, const float* Z, int64_t ldz, float* H, int64_t ldh, void* stream);
int gcn_relu_mask(int64_t rows, int32_t cols, const float* G, int64_t ldg, const float* Zprev,
                  int64_t ldzprev, float* out, int64_t ldo, void* stream);

/* -------------------------------------------------------------------------------------------
 * Last-layer activation and loss -- the row-wise log_softmax of "Block Two-Dimensional (2D)
 * Algorithms" with the mean negative log-likelihood over all n vertices, and Equation 1 for it:
 *   loss = -(1/n) sum_i log_softmax(Z[i,:])[y_i],  G[i,j] = (softmax(Z[i,:])[j] - [j == y_i]) / n.
 * Z: device n x C (ld ldz); labels: device int32[n] in [0,C); loss: device float (written);
 * G: device n x C (ld ldg) or NULL.  Row sums are reduced in double in a fixed order.
 * ----------------------------------------------------------------------------------------- */
int gcn_softmax_nll(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels, float* loss,
                    float* G, int64_t ldg, void* stream);

/* The same with a training split (the paper trains Reddit on a split, "Datasets and Compute
 * Platform"): vertices with a negative label are outside the split; they add nothing to the loss and
 * their rows of G are zero.  n_labelled = number of vertices with label >= 0 (host value, the caller
 * knows its split); the mean and the 1/n factor of G use it.  BADARG unless 1 <= n_labelled <= n. */
int gcn_softmax_nll_masked(int64_t n, int32_t C, const float* Z, int64_t ldz, const int32_t* labels,
                           int64_t n_labelled, float* loss, float* G, int64_t ldg, void* stream);

/* -------------------------------------------------------------------------------------------
 * One layer forward -- "Forward Propagation": Z = A^T Hin W (+ bias), Hout = sigma(Z).
 * Needs GCN_BUILD_TRANSPOSE.  Hin: n x f_in (ld ldh).  W: f_in x f_out dense.  Z, Hout: n x f_out
 * dense (Hout may be NULL with GCN_ACT_NONE, and may equal Z).  T: scratch, n x f_out dense for
 * GEMM_FIRST (holds Hin W), n x f_in dense for SPMM_FIRST (holds A^T Hin; keep it for backward).
 * ----------------------------------------------------------------------------------------- */
int gcn_layer_forward(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh,
                      const float* W, const float* bias, float* Z, float* Hout, float* T, int order,
                      int act, void* stream);

/* -------------------------------------------------------------------------------------------
 * One layer backward -- Equations 2 and 3 with A G computed once and used for both:
 *   Y = Hin^T A G            (f_in x f_out, gradient of W)
 *   Gprev = (A G W^T) (Hadamard) sigma'(Zprev)     (n x f_in; pass Gprev = NULL at the first layer)
 * G: n x f_out dense = dL/dZ of this layer.  dbias (f_out, column sums of G) may be NULL.
 * S: scratch, n x f_out for GEMM_FIRST (returns A G), n x f_in for SPMM_FIRST (returns G W^T).
 * T: the forward call's T; read only in SPMM_FIRST order (Y = T^T G).  `order` must be the order
 * the forward call resolved to (AUTO resolves identically in both).
 * ----------------------------------------------------------------------------------------- */
int gcn_layer_backward(gcn_csr* a, int32_t f_in, int32_t f_out, const float* Hin, int64_t ldh,
                       const float* Zprev, const float* W, const float* G, const float* T, float* S,
                       float* Y, float* dbias, float* Gprev, int order, void* stream);

/* -------------------------------------------------------------------------------------------
 * One full-batch epoch: forward through L_w layers (ReLU between, none after the last), loss,
 * backward, and W <- W - lr Y when lr != 0 (the gradient step of Equation 3).
 * dims: HOST int32[L_w+1] = f^0..f^{L_w}.  H0: device n x dims[0] dense.  labels: device int32[n].
 * W, Y: HOST arrays of L_w device pointers (W[l] is dims[l] x dims[l+1]; Y[l] receives dL/dW[l]).
 * loss: device float.  workspace: device, 256-byte aligned, at least gcn_epoch_workspace_bytes();
 * holds every H^l, Z^{L_w}, G^l, the scratch matrices and the partial sums of the reductions over n,
 * O(n * sum f).  `order` applies to every layer.
 * The first call with a given matrix, width set and configuration may build schedules and grow the handle's
 * buffers (device allocations, one wait for the stream) unless gcn_epoch_prepare ran before.  Otherwise the
 * call only enqueues kernels and device-to-device copies on `stream`, so it can be captured in a HIP graph
 * and replayed; all reductions run in a fixed order, so repeated epochs give bit-identical results.
 * ----------------------------------------------------------------------------------------- */
int gcn_epoch(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* H0, const int32_t* labels,
              float* const* W, float* const* Y, float lr, float* loss, void* workspace,
              size_t workspace_bytes, int order, void* stream);

/* gcn_epoch with a training split: labels < 0 mark vertices outside it, n_labelled counts the others
 * (see gcn_softmax_nll_masked).  Calling it in a loop with lr != 0 is full-batch gradient descent. */
/* gcn_spmm_prepare for every sparse product of an epoch with these arguments (both stored matrices, the widths
 * the association order gives).  After it, gcn_epoch* with the same matrix, dims and order only queues work. */
int gcn_epoch_prepare(gcn_csr* a, int32_t L_w, const int32_t* dims, int order, void* stream);

int gcn_epoch_masked(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* H0, const int32_t* labels,
                     int64_t n_labelled, float* const* W, float* const* Y, float lr, float* loss, void* workspace,
                     size_t workspace_bytes, int order, void* stream);

/* The same epoch for a caller that trains many epochs on fixed input features: "Forward Propagation"
 * computes Z^1 = (A^T H^0) W^1 and Equation 3 gives Y^1 = (A^T H^0)^T G^1, and A^T H^0 does not change
 * between epochs.  P0 (device, n x dims[0] dense) is that product, computed once by the caller with
 * gcn_spmm(a, 1, dims[0], H0, ...); the first layer then needs no sparse product in either direction.
 * Everything else (arguments, workspace, views, results up to fp32 summation order) as gcn_epoch_masked;
 * `order` applies to layers 2..L_w. */
int gcn_epoch_preaggregated(gcn_csr* a, int32_t L_w, const int32_t* dims, const float* P0, const int32_t* labels,
                            int64_t n_labelled, float* const* W, float* const* Y, float lr, float* loss,
                            void* workspace, size_t workspace_bytes, int order, void* stream);
size_t gcn_epoch_workspace_bytes(int64_t n, int32_t L_w, const int32_t* dims, int order);

/* After gcn_epoch: device pointers into the workspace for layer l in [1, L_w], both n x dims[l]
 * dense, for parity checks: G = G^l; Z = Z^l for the last layer and H^l = ReLU(Z^l) for the hidden
 * layers (their Z is never stored: sigma'(Z) = [H > 0]).  For the last layer see GCN_CFG_FUSED_LAST_LAYER: with the
 * fused last layer (the default where it applies) Z^L and G^L are stored only on request.  BADARG if l or the
 * workspace is bad. */
int gcn_epoch_view(int64_t n, int32_t L_w, const int32_t* dims, int order, void* workspace, int32_t l,
                   float** Z, float** G);

/* Process-wide settings (GCN_CFG_*), followed by every matrix that has no settings of its own.  Returns BADARG
 * for an unknown key or value.  gcn_csr_config gives one matrix its own settings: the first call copies the
 * process-wide ones into the matrix, which from then on ignores gcn_config (GCN_CFG_TIMING stays process-wide). */
int gcn_config(int key, int value);
int gcn_csr_config(gcn_csr* a, int key, int value);

/* Frees the library-owned per-stream scratch (after waiting for the device); later calls allocate it again. */
int gcn_scratch_release(void);

/* With GCN_CFG_TIMING = 1 the SpMM main kernel is bracketed by HIP events on its own stream.
 * gcn_timing_read synchronises with the recorded events, returns the number of bracketed
 * launches and their total milliseconds since the last read, and resets the record.
 * The layer and epoch calls also bracket their phases: gcn_timing_read_phases fills
 * spans[GCN_PHASE_COUNT] and total_ms[GCN_PHASE_COUNT] (host arrays) and resets the record:
 *   GCN_PHASE_SPMM_KERNEL  the SpMM main kernels alone (what gcn_timing_read returns)
 *   GCN_PHASE_SPMM         whole sparse products (pre-scaling, main, fix-up and reduce kernels)
 *   GCN_PHASE_GEMM         dense products
 *   GCN_PHASE_OTHER        loss, activation, bias and update kernels */
#define GCN_PHASE_SPMM_KERNEL 0
#define GCN_PHASE_SPMM 1
#define GCN_PHASE_GEMM 2
#define GCN_PHASE_OTHER 3
#define GCN_PHASE_COUNT 4
int gcn_timing_read(int64_t* launches, double* total_ms);
int gcn_timing_read_phases(int64_t* spans, double* total_ms);

/* Building blocks of graph construction (section "Graph Neural Networks": the modified adjacency matrix
 * is assembled from an edge list; gcn_csr_create sorts 64-bit keys row<<32|col, drops equal neighbours and
 * takes prefix sums with exactly these routines).  Exported so that they can be checked on their own.  All
 * pointers are DEVICE pointers, inputs are left unchanged, outputs must not overlap inputs (gcn_exclusive_scan_i64
 * allows in == out); the calls allocate temporaries on the device and return after the stream has finished.
 *
 * gcn_radix_sort: stable sort of n keys of key_bytes (4 or 8: unsigned) by their bits [0, end_bit), ascending or
 * descending (descending != 0); equal keys keep their input order.  payload_bytes 0, 4, 8 or 12: a payload record
 * of that size moves with each key (payload pointers NULL when 0).  GCN_ERR_BADARG for other sizes.
 * gcn_exclusive_scan_i64: out[i] = in[0] + ... + in[i-1] (out[0] = 0), 64-bit wrap-around arithmetic.
 * gcn_unique_u64: keeps the first key of every run of equal neighbours, in order; *count (HOST pointer) receives
 * how many were kept. */
int gcn_radix_sort(int64_t n, int key_bytes, const void* keys_in, void* keys_out, int payload_bytes,
                   const void* payload_in, void* payload_out, int end_bit, int descending, void* stream);
int gcn_exclusive_scan_i64(int64_t n, const int64_t* in, int64_t* out, void* stream);
int gcn_unique_u64(int64_t n, const uint64_t* keys_in, uint64_t* keys_out, int64_t* count, void* stream);

/* Which schedule the most recent sparse product of this process took (for tests and reports; not
 * meaningful while several threads run products). */
#define GCN_SCHED_ROWWISE 1
#define GCN_SCHED_SPLIT 2    /* nonzero-split over the stored order */
#define GCN_SCHED_SWEEP 3    /* column sweep (+ nonzero-split for its long rows) */
#define GCN_SCHED_HUB 4      /* hub schedule */
#define GCN_SCHED_BLOCKED 5  /* nonzero-split over the column-blocked copy */
int gcn_last_spmm_schedule(void);
int gcn_csr_last_spmm_schedule(const gcn_csr* a);   /* the same per matrix (0 before its first product) */
/* Number of stored orders of matrices (column-blocked, sweep, hub copies) this process has built so far: a
 * caller can check that a steady-state loop builds nothing. */
int64_t gcn_build_count(void);

const char* gcn_last_error(void);
const char* gcn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GCN_H */
