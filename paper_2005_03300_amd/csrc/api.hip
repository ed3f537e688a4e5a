// Error reporting, settings, event timing, allocation helpers and gcn_csr accessors.
#include <stdarg.h>
#include <string.h>

#include <atomic>
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

// ---- per-stream scratch ------------------------------------------------------------------------
struct Arena { int device; hipStream_t stream; void* p; size_t bytes; };
static std::mutex g_scratch_mu;
static std::vector<Arena> g_arenas;
static std::vector<void*> g_scratch_retired;

static thread_local void* g_scope_p = nullptr;
static thread_local size_t g_scope_bytes = 0;

ScratchScope::ScratchScope(void* p, size_t bytes) : prev_p(g_scope_p), prev_bytes(g_scope_bytes) {
    g_scope_p = p;
    g_scope_bytes = bytes;
}
ScratchScope::~ScratchScope() {
    g_scope_p = prev_p;
    g_scope_bytes = prev_bytes;
}

int scratch_get(void** p, size_t bytes, hipStream_t s) {
    if (g_scope_p) {
        if (bytes > g_scope_bytes)
            return fail(GCN_ERR_WORKSPACE, "workspace scratch region has %zu bytes, %zu needed", g_scope_bytes, bytes);
        *p = g_scope_p;
        return GCN_OK;
    }
    int dev = 0;
    GCN_HIP_TRY(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    Arena* ar = nullptr;
    for (auto& x : g_arenas)
        if (x.device == dev && x.stream == s) { ar = &x; break; }
    if (!ar) {
        g_arenas.push_back({dev, s, nullptr, 0});
        ar = &g_arenas.back();
    }
    if (bytes > ar->bytes) {
        // Work queued (or captured in a graph) earlier may still use the old buffer: keep it.
        void* fresh = nullptr;
        const size_t want = bytes + bytes / 4;
        GCN_TRY(device_alloc(&fresh, want));
        if (ar->p) g_scratch_retired.push_back(ar->p);
        ar->p = fresh;
        ar->bytes = want;
    }
    *p = ar->p;
    return GCN_OK;
}

int grow_retire(gcn_csr* a, float** buf, size_t* have, size_t need) {
    if (need <= *have) return GCN_OK;
    void* fresh = nullptr;
    GCN_TRY(device_alloc(&fresh, need));
    if (*buf) a->retired.push_back(*buf);
    *buf = (float*)fresh;
    *have = need;
    return GCN_OK;
}

const DeviceInfo& device_info() {
    static std::mutex mu;
    static DeviceInfo info[64];
    static bool known[64] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    if (dev < 0 || dev >= 64) dev = 0;
    std::lock_guard<std::mutex> lk(mu);
    if (!known[dev]) {
        int cus = 0, l2 = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        if (hipDeviceGetAttribute(&l2, hipDeviceAttributeL2CacheSize, dev) != hipSuccess || l2 <= 0) l2 = 4 << 20;
        info[dev] = {cus, (int64_t)l2};
        known[dev] = true;
    }
    return info[dev];
}

Config& config() {
    static Config c;
    return c;
}

int g_last_schedule = 0;

static std::atomic<int64_t> g_builds{0};
void count_build() { g_builds.fetch_add(1); }

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
    for (auto& b : m.blk_parked) free_blocked(b);
    for (auto& w : m.swp_parked) free_sweep(w);
    for (auto& h : m.hub_parked) free_hub(h);
    m = Matrix();
}

}  // namespace gcn

using namespace gcn;

extern "C" {

const char* gcn_last_error(void) { return g_err; }
const char* gcn_version(void) { return "gcn-hip 0.1 (gfx950)"; }

int gcn_last_spmm_schedule(void) { return gcn::g_last_schedule; }

static int set_config(Config& c, int key, int value) {
    switch (key) {
        case GCN_CFG_SPMM_ALGO:
            if (value < 0 || value > 4) return fail(GCN_ERR_BADARG, "GCN_CFG_SPMM_ALGO must be 0, 1, 2, 3 or 4");
            c.spmm_algo = value;
            return GCN_OK;
        case GCN_CFG_SPMM_BLOCKS:
            if (value < 0 || value > (1 << 24)) return fail(GCN_ERR_BADARG, "GCN_CFG_SPMM_BLOCKS must be in [0, 2^24]");
            c.spmm_blocks = value;
            return GCN_OK;
        case GCN_CFG_SPLIT_LDS_KB:
            if (value < 18 || value > 64) return fail(GCN_ERR_BADARG, "GCN_CFG_SPLIT_LDS_KB must be in [18, 64]");
            c.split_lds_kb = value;
            return GCN_OK;
        case GCN_CFG_SWEEP_WAVES:
            if (value < 1 || value > 18) return fail(GCN_ERR_BADARG, "GCN_CFG_SWEEP_WAVES must be in [1, 18]");
            c.sweep_waves = value;
            return GCN_OK;
        case GCN_CFG_SWEEP_HEAVY:
            if (value < 1) return fail(GCN_ERR_BADARG, "GCN_CFG_SWEEP_HEAVY must be at least 1");
            c.sweep_heavy = value;
            return GCN_OK;
        case GCN_CFG_HUB_MB:
            if (value < 1 || value > 4096) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_MB must be in [1, 4096]");
            c.hub_mb = value;
            return GCN_OK;
        case GCN_CFG_HUB_BLOCK_COLS:
            if (value < 0 || (value % 64) != 0) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_BLOCK_COLS must be 0 or a multiple of 64");
            c.hub_block_cols = value;
            return GCN_OK;
        case GCN_CFG_HUB_DMIN:
            if (value < 1) return fail(GCN_ERR_BADARG, "GCN_CFG_HUB_DMIN must be at least 1");
            c.hub_dmin = value;
            return GCN_OK;
        case GCN_CFG_PATTERN_SPMM:
            if (value < 0 || value > 2) return fail(GCN_ERR_BADARG, "GCN_CFG_PATTERN_SPMM must be 0, 1 or 2");
            c.pattern_spmm = value;
            return GCN_OK;
        case GCN_CFG_FUSED_LAST_LAYER:
            if (value < 0 || value > 2) return fail(GCN_ERR_BADARG, "GCN_CFG_FUSED_LAST_LAYER must be 0, 1 or 2");
            c.fused_last = value;
            return GCN_OK;
        case GCN_CFG_TIMING:
            if (value != 0 && value != 1) return fail(GCN_ERR_BADARG, "GCN_CFG_TIMING must be 0 or 1");
            c.timing = value;
            return GCN_OK;
        default:
            return fail(GCN_ERR_BADARG, "unknown config key %d", key);
    }
}

int gcn_config(int key, int value) { return set_config(config(), key, value); }

int gcn_csr_config(gcn_csr* a, int key, int value) {
    if (!a) return fail(GCN_ERR_BADARG, "gcn_csr_config: NULL matrix");
    if (key == GCN_CFG_TIMING) return fail(GCN_ERR_BADARG, "gcn_csr_config: GCN_CFG_TIMING is process-wide (gcn_config)");
    if (!a->own_cfg) {               // from now on this matrix no longer follows gcn_config
        a->cfg = config();
        a->own_cfg = true;
    }
    return set_config(a->cfg, key, value);
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
    device_free(a->xs);
    for (void* p : a->retired) device_free(p);
    delete a;
    return GCN_OK;
}

int gcn_scratch_release(void) {
    GCN_HIP_TRY(hipDeviceSynchronize());
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    for (auto& x : g_arenas) device_free(x.p);
    for (void* p : g_scratch_retired) device_free(p);
    g_arenas.clear();
    g_scratch_retired.clear();
    return GCN_OK;
}

int64_t gcn_build_count(void) { return g_builds.load(); }

int gcn_csr_last_spmm_schedule(const gcn_csr* a) { return a ? a->last_schedule : 0; }

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
