// Error reporting, settings, event timing, allocation helpers and gcn_csr accessors.
#include <stdarg.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "common.h"

namespace gcn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int device_alloc(void** p, size_t bytes) {
    *p = nullptr;
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        return fail(e == hipErrorOutOfMemory ? GCN_ERR_OOM : GCN_ERR_HIP, "hipMalloc(%zu) failed: %s", bytes,
                    hipGetErrorString(e));
    }
    return GCN_OK;
}

void device_free(void* p) {
    if (p) (void)hipFree(p);
}

static std::mutex g_scratch_mu;
static void* g_scratch = nullptr;
static size_t g_scratch_bytes = 0;

int scratch_get(void** p, size_t bytes) {
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (bytes > g_scratch_bytes) {
        // Work queued earlier may still read the old buffer: wait before freeing it.
        if (g_scratch) {
            GCN_HIP_TRY(hipDeviceSynchronize());
            device_free(g_scratch);
            g_scratch = nullptr;
            g_scratch_bytes = 0;
        }
        size_t want = bytes + bytes / 4;
        GCN_TRY(device_alloc(&g_scratch, want));
        g_scratch_bytes = want;
    }
    *p = g_scratch;
    return GCN_OK;
}

Config& config() {
    static Config c;
    return c;
}

int g_last_schedule = 0;

// ---- event timing ---------------------------------------------------------------------------
struct TimedSpan { hipEvent_t a, b; int phase; };
static std::mutex g_time_mu;
static std::vector<TimedSpan> g_events;
static thread_local hipEvent_t g_open[GCN_PHASE_COUNT] = {};

void timing_begin(hipStream_t s, int phase) {
    if (!config().timing || g_open[phase]) return;
    hipEvent_t a;
    if (hipEventCreate(&a) != hipSuccess) return;
    (void)hipEventRecord(a, s);
    g_open[phase] = a;
}

void timing_end(hipStream_t s, int phase) {
    if (!g_open[phase]) return;
    hipEvent_t b;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(g_open[phase]);
        g_open[phase] = nullptr;
        return;
    }
    (void)hipEventRecord(b, s);
    std::lock_guard<std::mutex> lk(g_time_mu);
    g_events.push_back({g_open[phase], b, phase});
    g_open[phase] = nullptr;
}

void free_blocked(Blocked& b) {
    device_free(b.colidx);
    device_free(b.val);
    device_free(b.flags);
    device_free(b.sub_row);
    device_free(b.rp);
    device_free(b.fix_list);
    device_free(b.rq_ptr);
    device_free(b.rq_idx);
    b = Blocked();
}

void free_matrix(Matrix& m);

void free_sweep(Sweep& w) {
    device_free(w.colidx);
    device_free(w.val);
    device_free(w.lrow);
    device_free(w.task_base);
    device_free(w.task_len);
    device_free(w.task_order);
    if (w.heavy) {
        free_matrix(*w.heavy);
        delete w.heavy;
    }
    w = Sweep();
}

void free_hub(Hub& h) {
    device_free(h.hot_col);
    device_free(h.heavy_rows);
    device_free(h.defer);
    device_free(h.xhot);
    if (h.hot) { free_matrix(*h.hot); delete h.hot; }
    if (h.rest) { free_matrix(*h.rest); delete h.rest; }
    h = Hub();
}

void free_matrix(Matrix& m) {
    device_free(m.rowptr);
    device_free(m.colidx);
    device_free(m.val);
    device_free(m.flags);
    device_free(m.sub_row);
    device_free(m.ne_rows);
    device_free(m.ne_rowptr);
    device_free(m.empty_rows);
    device_free(m.fix_list);
    free_blocked(m.blk);
    free_sweep(m.swp);
    free_hub(m.hub);
    m = Matrix();
}

}  // namespace gcn

using namespace gcn;

extern "C" {

const char* gcn_last_error(void) { return g_err; }
const char* gcn_version(void) { return "gcn-hip 0.1 (gfx950)"; }

int gcn_last_spmm_schedule(void) { return gcn::g_last_schedule; }

int gcn_config(int key, int value) {
    switch (key) {
        case GCN_CFG_SPMM_ALGO:
            if (value < 0 || value > 4) return fail(GCN_ERR_BADARG, "GCN_CFG_SPMM_ALGO must be 0, 1, 2, 3 or 4");
            config().spmm_algo = value;
            return GCN_OK;
        case GCN_CFG_SPMM_BLOCKS:
            if (value < 0 || value > (1 << 24)) return fail(GCN_ERR_BADARG, "GCN_CFG_SPMM_BLOCKS must be in [0, 2^24]");
            config().spmm_blocks = value;
            return GCN_OK;
        case GCN_CFG_SPLIT_LDS_KB:
            if (value < 18 || value > 64) return fail(GCN_ERR_BADARG, "GCN_CFG_SPLIT_LDS_KB must be in [18, 64]");
            config().split_lds_kb = value;
            return GCN_OK;
        case GCN_CFG_SWEEP_WAVES:
            if (value < 1 || value > 18) return fail(GCN_ERR_BADARG, "GCN_CFG_SWEEP_WAVES must be in [1, 18]");
            config().sweep_waves = value;
            return GCN_OK;
        case GCN_CFG_SWEEP_HEAVY:
            if (value < 1) return fail(GCN_ERR_BADARG, "GCN_CFG_SWEEP_HEAVY must be at least 1");
            config().sweep_heavy = value;
            return GCN_OK;
        case GCN_CFG_HUB_MB:
            if (value < 1 || value > 4096) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_MB must be in [1, 4096]");
            config().hub_mb = value;
            return GCN_OK;
        case GCN_CFG_HUB_BLOCK_COLS:
            if (value < 0 || (value % 64) != 0) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_BLOCK_COLS must be 0 or a multiple of 64");
            config().hub_block_cols = value;
            return GCN_OK;
        case GCN_CFG_HUB_DMIN:
            if (value < 1) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_DMIN must be at least 1");
            config().hub_dmin = value;
            return GCN_OK;
        case GCN_CFG_PATTERN_SPMM:
            if (value < 0 || value > 2) return fail(GCN_ERR_BADARG, "GCN_CFG_PATTERN_SPMM must be 0, 1 or 2");
            config().pattern_spmm = value;
            return GCN_OK;
        case GCN_CFG_TIMING:
            if (value != 0 && value != 1) return fail(GCN_ERR_BADARG, "GCN_CFG_TIMING must be 0 or 1");
            config().timing = value;
            return GCN_OK;
        default:
            return fail(GCN_ERR_BADARG, "unknown config key %d", key);
    }
}

int gcn_timing_read_phases(int64_t* spans, double* total_ms) {
    if (!spans || !total_ms) return fail(GCN_ERR_BADARG, "gcn_timing_read_phases: NULL output");
    std::lock_guard<std::mutex> lk(g_time_mu);
    for (int p = 0; p < GCN_PHASE_COUNT; ++p) { spans[p] = 0; total_ms[p] = 0.0; }
    int rc = GCN_OK;
    for (auto& ev : g_events) {
        float t = 0.f;
        hipError_t e = hipEventSynchronize(ev.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, ev.a, ev.b);
        if (e == hipSuccess) {
            total_ms[ev.phase] += t;
            spans[ev.phase] += 1;
        } else {
            rc = fail(GCN_ERR_HIP, "event timing failed: %s", hipGetErrorString(e));
        }
        (void)hipEventDestroy(ev.a);
        (void)hipEventDestroy(ev.b);
    }
    g_events.clear();
    return rc;
}

int gcn_timing_read(int64_t* launches, double* total_ms) {
    if (!launches || !total_ms) return fail(GCN_ERR_BADARG, "gcn_timing_read: NULL output");
    int64_t spans[GCN_PHASE_COUNT];
    double ms[GCN_PHASE_COUNT];
    const int rc = gcn_timing_read_phases(spans, ms);
    *launches = spans[GCN_PHASE_SPMM_KERNEL];
    *total_ms = ms[GCN_PHASE_SPMM_KERNEL];
    return rc;
}

int gcn_csr_destroy(gcn_csr* a) {
    if (!a) return GCN_OK;
    (void)hipDeviceSynchronize();
    free_matrix(a->A);
    free_matrix(a->At);
    device_free(a->carry2);
    device_free(a->deg);
    device_free(a->inv_sqrt_deg);
    device_free(a->carry);
    device_free(a->partial);
    delete a;
    return GCN_OK;
}

int gcn_csr_info(const gcn_csr* a, int64_t* n, int64_t* nnz, int32_t* max_degree) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_csr_info: NULL matrix");
    if (n) *n = a->n;
    if (nnz) *nnz = a->nnz;
    if (max_degree) *max_degree = a->A.max_degree;
    return GCN_OK;
}

int gcn_csr_shape(const gcn_csr* a, int64_t* n_rows, int64_t* n_cols) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_csr_shape: NULL matrix");
    if (n_rows) *n_rows = a->n;
    if (n_cols) *n_cols = a->ncols;
    return GCN_OK;
}

int gcn_csr_arrays(const gcn_csr* a, int transposed, const int64_t** rowptr, const int32_t** colidx,
                   const float** val, const int32_t** deg) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_csr_arrays: NULL matrix");
    if (transposed && !a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "matrix was built without GCN_BUILD_TRANSPOSE");
    const Matrix& m = transposed ? a->At : a->A;
    if (rowptr) *rowptr = m.rowptr;
    if (colidx) *colidx = m.colidx;
    if (val) *val = m.val;
    if (deg) *deg = a->deg;
    return GCN_OK;
}

int gcn_csr_export(const gcn_csr* a, int transposed, int64_t* rowptr, int32_t* colidx, float* val, int32_t* deg,
                   void* stream) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_csr_export: NULL matrix");
    if (transposed && !a->has_t) return fail(GCN_ERR_NOTRANSPOSE, "matrix was built without GCN_BUILD_TRANSPOSE");
    const Matrix& m = transposed ? a->At : a->A;
    hipStream_t s = (hipStream_t)stream;
    if (rowptr) GCN_HIP_TRY(hipMemcpyAsync(rowptr, m.rowptr, ((size_t)m.nrows + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, s));
    if (colidx && a->nnz) GCN_HIP_TRY(hipMemcpyAsync(colidx, m.colidx, (size_t)a->nnz * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    if (val && a->nnz) GCN_HIP_TRY(hipMemcpyAsync(val, m.val, (size_t)a->nnz * sizeof(float), hipMemcpyDeviceToDevice, s));
    if (deg) GCN_HIP_TRY(hipMemcpyAsync(deg, a->deg, (size_t)a->n * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
    return GCN_OK;
}

}  // extern "C"
