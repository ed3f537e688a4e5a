// Internal declarations shared by the translation units of libgcn_hip.so (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <string>
#include <vector>

#include "gcn.h"

namespace gcn {

// Thread-local error text returned by gcn_last_error().
void set_error(const char* fmt, ...);
int fail(int code, const char* fmt, ...);

#define GCN_HIP_TRY(expr)                                                                       \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess)                                                                   \
            return gcn::fail(e_ == hipErrorOutOfMemory ? GCN_ERR_OOM : GCN_ERR_HIP,             \
                             "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__,   \
                             __LINE__);                                                         \
    } while (0)

#define GCN_TRY(expr)          \
    do {                       \
        int rc_ = (expr);      \
        if (rc_ != GCN_OK) return rc_; \
    } while (0)

// Launch check: a bad configuration is reported by hipGetLastError right after the launch.
#define GCN_LAUNCH_CHECK()                                                                      \
    do {                                                                                        \
        hipError_t e_ = hipGetLastError();                                                      \
        if (e_ != hipSuccess)                                                                   \
            return gcn::fail(GCN_ERR_HIP, "kernel launch failed: %s (%s:%d)",                   \
                             hipGetErrorString(e_), __FILE__, __LINE__);                        \
    } while (0)

// Nonzero-split schedule constants: a wavefront owns CHUNK consecutive stored entries, cut into
// SUB-entry pieces that each carry one 32-bit word of row-start flags.
constexpr int SUB = 32;
constexpr int CHUNK = 512;
constexpr int SUBS_PER_CHUNK = CHUNK / SUB;

// Column-blocked copy of a matrix: the entries re-sorted by (column block, row, column).  Each
// non-empty (block, row) pair is a row of a partial-result matrix P; the SpMM kernel runs over this
// order unchanged, so all wavefronts gather from one block of X at a time and that block stays in
// L2.  A second kernel adds each row's partials in ascending block order.
struct Blocked {
    int64_t cols_per_block = 0;
    int32_t nblocks = 0;
    int64_t nrows = 0;           // R: non-empty (block, row) pairs
    int32_t* colidx = nullptr;   // [nnz]
    float* val = nullptr;        // [nnz]
    uint32_t* flags = nullptr;   // [nsub + pad]
    int32_t* sub_row = nullptr;  // [nsub + pad]
    int64_t* rp = nullptr;       // [R+1] first entry of each partial row
    int32_t* fix_list = nullptr; // [n_fix] chunks that lead the continuation of a row begun in an earlier chunk
    int64_t n_fix = -1;          // -1: no list (every chunk is examined)
    int64_t* rq_ptr = nullptr;   // [n+1]  row i owns partial rows rq_idx[rq_ptr[i] .. rq_ptr[i+1])
    int32_t* rq_idx = nullptr;   // [R]    ascending block order inside a row
};

struct Matrix;

// Sweep copy of a matrix for operands far larger than the caches.  Rows are cut into tasks of
// `rb` consecutive rows; a wavefront owns a task, accumulates its rows in LDS and walks the task's
// entries in ascending column order, so all wavefronts of a launch (started together, equal length)
// gather from one narrow band of X at a time and that band stays in L2.  The entries of a task are
// stored in steps of `groups` entries whose rows all differ (packed that way when the copy is built,
// an entry whose row is already in the step moving to one of the next steps), so the lane groups of
// one step add to LDS without any conflict; padding entries have column -1.  Rows longer than
// `heavy_threshold` are kept apart and go through the nonzero-split kernel.
struct Sweep {
    int32_t groups = 0;
    int32_t rb = 0;
    int32_t heavy_threshold = 0;
    int64_t ntasks = 0, nnz_light = 0, nnz_heavy = 0, n_heavy = 0;
    int64_t padded = 0;           // entries stored, padding included
    int32_t* colidx = nullptr;    // [padded] column, or -1 for a padding entry
    float* val = nullptr;         // [padded]
    uint8_t* lrow = nullptr;      // [padded] row inside the task
    int64_t* task_base = nullptr; // [ntasks] first stored entry of the task (multiple of 16)
    int32_t* task_len = nullptr;  // [ntasks] stored entries of the task (multiple of groups)
    int32_t* task_order = nullptr;// [ntasks] task ids, longest first
    Matrix* heavy = nullptr;      // the heavy rows as a row-subset matrix (ne_rows = their ids)
};

// Hub copy of a matrix with a skewed degree distribution: A = A_hot + A_rest, where A_hot holds the
// entries of long rows (at least `dmin` entries) whose column is one of the `H` columns with the most
// entries, and A_rest everything else.  The rows of X that the hot columns select are packed, in
// descending order of column length, into a buffer of their own at every product; A_hot runs over it
// in column blocks that stay in one L2 each (every XCD works on its own blocks), A_rest runs over X
// unchanged, and the partial rows of A_hot are added to the rows that A_rest wrote.
struct Hub {
    int state = 0;                // 0 not tried, 1 built, -1 tried and rejected (not skewed enough)
    int64_t H = 0, cpb = 0;       // hot columns, columns per block (H is a multiple of cpb)
    int32_t dmin = 0;
    int32_t cfg_mb = 0, cfg_block_cols = 0;   // settings at build time: a change of settings rebuilds, a change of f does not
    int64_t nnz_hot = 0, nnz_rest = 0, n_heavy = 0;
    int32_t* hot_col = nullptr;   // [H] position in the packed buffer -> column
    int32_t* heavy_rows = nullptr;// [n_heavy] the long rows, ascending
    uint8_t* defer = nullptr;     // [nrows] 1 for a long row: A_rest stores its sum raw, A_hot's pass finishes it
    Matrix* hot = nullptr;        // n_heavy x H, column = position in the packed buffer
    Matrix* rest = nullptr;       // nrows x ncols
    float* xhot = nullptr;        // [H][f] packed rows of X, grown on demand
    size_t xhot_bytes = 0;
};

// One stored matrix in compressed rows plus its nonzero-split schedule.
struct Matrix {
    int64_t nrows = 0, ncols = 0;
    int64_t* rowptr = nullptr;   // [nrows+1]
    int32_t* colidx = nullptr;   // [nnz]
    float* val = nullptr;        // [nnz]
    // schedule (built once at creation)
    uint32_t* flags = nullptr;   // [nsub]  bit b of word j: entry 32j+b is the first of its row
    int32_t* sub_row = nullptr;  // [nsub]  index (among non-empty rows) of the row holding entry 32j
    int32_t* ne_rows = nullptr;  // [n_ne]  non-empty row index -> row, or NULL when no row is empty
    int64_t* ne_rowptr = nullptr;// [n_ne+1] rowptr restricted to non-empty rows, or NULL (= rowptr)
    int32_t* empty_rows = nullptr;// [nrows - n_ne] the rows without entries, or NULL when there are none
    int64_t n_ne = 0;
    int32_t* fix_list = nullptr; // [n_fix] chunks that lead the continuation of a row begun in an earlier chunk
    int64_t n_fix = -1;          // -1: no list (every chunk is examined)
    int64_t nsub = 0, nchunks = 0;
    int32_t max_degree = 0;
    // Other stored orders of the matrix, built on first use (or by a prepare call) and kept until the
    // matrix is destroyed.  blk / swp / hub are the copies the latest product used; a product that needs
    // another key (block width; lane groups, task height and long-row threshold; hub settings) parks the
    // current copy in the list beside it and takes the matching one from there, or builds it.  Nothing is
    // freed before destroy, so kernels already queued (or captured in a HIP graph) keep valid pointers.
    Blocked blk;
    Sweep swp;
    Hub hub;
    std::vector<Blocked> blk_parked;
    std::vector<Sweep> swp_parked;
    std::vector<Hub> hub_parked;
};

struct Config {
    int spmm_algo = 0;
    int spmm_blocks = 0;
    int sweep_heavy = 1024;
    int split_lds_kb = 28;       // nonzero-split kernels for rows of up to 64 bytes: LDS per workgroup incl. padding (18: none)
    int sweep_waves = 9;
    int hub_mb = 32;             // hub schedule: size of the packed buffer of hot rows of X, MB
    int hub_block_cols = 0;      // hub schedule: columns per block (0: about 2 MB of the gathered panel)
    int hub_dmin = 64;           // hub schedule: rows with at least this many entries are long rows
    int pattern_spmm = 2;        // epoch: value-free SpMM for symmetric normalisation (0 never, 1 always, 2 by row length)
    int fused_last = 1;          // epoch: fused last layer (0 off, 1 on without storing Z^L and G^L, 2 on and stored)
    int timing = 0;
};

}  // namespace gcn

struct gcn_csr {
    int64_t n = 0, ncols = 0, nnz = 0;   // A is n x ncols (square unless made by gcn_csr_create_from_csr_rect)
    int device = 0;
    bool has_t = false;
    gcn::Matrix A, At;
    int32_t* deg = nullptr;      // [n] entries per row of A
    float* inv_sqrt_deg = nullptr; // [n] (float)(1/sqrt(deg)); set only when this library normalised the matrix
                                 // symmetrically, i.e. val_ij == 1/sqrt(deg_i deg_j) for every stored entry
    float* carry = nullptr;      // per-chunk partial rows for the nonzero-split SpMM
    size_t carry_bytes = 0;
    float* carry2 = nullptr;     // the same for the second matrix of a paired launch
    size_t carry2_bytes = 0;
    float* partial = nullptr;    // P of the column-blocked SpMM
    size_t partial_bytes = 0;
    float* xs = nullptr;         // operand of gcn_spmm with its rows pre-scaled (value-free form)
    size_t xs_bytes = 0;
    std::vector<void*> retired;  // buffers replaced by larger ones: kept until destroy (queued or captured work may use them)
    bool own_cfg = false;        // set by gcn_csr_config: this matrix has settings of its own
    gcn::Config cfg;             // valid when own_cfg
    int last_schedule = 0;       // GCN_SCHED_* of the latest product on this matrix
};

namespace gcn {

int device_alloc(void** p, size_t bytes);
template <typename T>
int device_alloc_t(T** p, size_t count) { return device_alloc((void**)p, count * sizeof(T)); }
void device_free(void* p);

// Library-owned scratch for the split-K partial sums of the weight-gradient product, the column sums and the
// loss: one buffer per (device, stream), so calls on different streams never share it.  It grows on demand; the
// buffer it replaces is kept (work queued or captured earlier may still use it) until gcn_scratch_release.
int scratch_get(void** p, size_t bytes, hipStream_t s);
// While one of these is alive on a thread, scratch_get on that thread hands out the given caller-owned
// buffer instead (GCN_ERR_WORKSPACE if it is too small): the epoch calls keep their partial sums in the
// caller's workspace.
struct ScratchScope {
    ScratchScope(void* p, size_t bytes);
    ~ScratchScope();
    void* prev_p;
    size_t prev_bytes;
};
// bytes of that scratch the split-K product (ta = 1) and the column sums take for the given shape
size_t gemm_tn_scratch_bytes(int64_t M, int64_t N, int64_t K);
size_t colsum_scratch_bytes(int64_t rows, int32_t cols);
size_t loss_scratch_bytes();

// Compute units and L2 size (one XCD's) of the current device, read once per device from the runtime.
struct DeviceInfo { int cus; int64_t l2_bytes; };
const DeviceInfo& device_info();

Config& config();                               // the process-wide settings (gcn_config)
inline const Config& cfg_of(const gcn_csr* a) { return a->own_cfg ? a->cfg : config(); }
// schedule taken by the most recent sparse product of this process (GCN_SCHED_*), for tests and reports
extern int g_last_schedule;
void count_build();

// event bracketing of the dominant kernel (GCN_CFG_TIMING)
void timing_begin(hipStream_t s, int phase = GCN_PHASE_SPMM_KERNEL);
void timing_end(hipStream_t s, int phase = GCN_PHASE_SPMM_KERNEL);
// brackets a scope of host code (all kernels it queues on `s`) under one phase
struct PhaseTimer {
    hipStream_t s;
    int phase;
    PhaseTimer(hipStream_t s_, int phase_) : s(s_), phase(phase_) { timing_begin(s, phase); }
    ~PhaseTimer() { timing_end(s, phase); }
};

int build_schedule(Matrix& m, int64_t n, int64_t nnz, hipStream_t s);
int build_fix_list(const uint32_t* flags, const int32_t* sub_row, const int64_t* rp, int64_t nchunks, int32_t** list,
                   int64_t* count, hipStream_t s);
int build_blocked(Matrix& m, int64_t nnz, int64_t cols_per_block, hipStream_t s);
// make m.blk / m.swp the copy with the given key: the current one, a parked one, or a newly built one
int want_blocked(Matrix& m, int64_t nnz, int64_t cols_per_block, hipStream_t s);
int want_sweep(Matrix& m, int64_t nnz, int32_t groups, int32_t rb, int32_t heavy_threshold, hipStream_t s);
void free_blocked(Blocked& b);
int build_sweep(Matrix& m, int64_t nnz, int32_t groups, int32_t rb, int32_t heavy_threshold, hipStream_t s);
void free_sweep(Sweep& w);
int build_hub(Matrix& m, int64_t nnz, int64_t H, int64_t cpb, int32_t dmin, hipStream_t s);
void free_hub(Hub& h);
void free_matrix(Matrix& m);

// Variants of the sparse product: `pattern` ignores the stored values (every entry counts as 1),
// `row_scale` multiplies output row i by row_scale[i] before the epilogue.
struct SpmmOpt {
    bool pattern = false;
    const float* row_scale = nullptr;
    // internal to the hub schedule:
    const uint8_t* defer = nullptr;   // rows whose sum is stored raw (no scale, no epilogue)
    bool accumulate = false;          // column-blocked reduce adds to what Z already holds
    // prepare / describe:
    bool dry = false;                 // build the stored order and size the buffers, launch nothing
    std::string* describe = nullptr;  // receives the schedule and its launch shape as text
};
int scale_rows_launch(int64_t rows, int32_t cols, const float* X, int64_t ldx, const float* scale, float* Y, int64_t ldy,
                      hipStream_t s);
// whether products with this matrix take the value-free form (GCN_CFG_PATTERN_SPMM and the matrix's own shape)
bool use_value_free(const gcn_csr* a);
int inv_sqrt_deg_launch(int64_t n, const int32_t* deg, float* out, hipStream_t s);
int spmm_launch(gcn_csr* a, Matrix& m, int32_t f, const float* X, int64_t ldx, float* Z, int64_t ldz,
                int epilogue, const float* Zprev, int64_t ldzprev, hipStream_t s, const SpmmOpt& o = SpmmOpt());
// builds the stored order and sizes the handle's buffers that spmm_launch would need for width f (16-byte
// aligned operands with leading dimensions that are multiples of 4 assumed), without running the product
int spmm_prepare(gcn_csr* a, Matrix& m, int32_t f, hipStream_t s);
// grows one of the handle's buffers; the replaced buffer is retired, not freed
int grow_retire(gcn_csr* a, float** buf, size_t* have, size_t need);

// `row_scale` (optional): row i of C is multiplied by row_scale[i] after bias and epilogue
int gemm_launch(int ta, int tb, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda, const float* B,
                int64_t ldb, float* C, int64_t ldc, const float* bias, int epilogue, const float* Zprev,
                int64_t ldzprev, hipStream_t s, const float* row_scale = nullptr);
// the fused last layer of the epoch (f_in = 16, up to 256 classes)
bool fused_last_supported(int32_t f_in, int32_t C);
size_t fused_last_scratch_bytes(int64_t n, int32_t C);
int fused_last_launch(int64_t n, int32_t C, const float* T, const float* W, const int32_t* labels, int64_t n_labelled,
                      float* loss, float* Y, float* S, const float* s_scale, float* Zout, float* Gout, void* scratch,
                      hipStream_t s);
int colsum_launch(int64_t rows, int32_t cols, const float* G, int64_t ldg, float* out, hipStream_t s);
int axpy_launch(int64_t count, float* W, const float* Y, float lr, hipStream_t s);
int relu_launch(int64_t rows, int32_t cols, const float* Z, int64_t ldz, float* H, int64_t ldh, hipStream_t s);
int bias_add_launch(int64_t rows, int32_t cols, float* Z, int64_t ldz, const float* bias, int relu, hipStream_t s);

}  // namespace gcn
