// Graph construction on the GPU: cleaned entry set -> compressed rows, degrees, normalised
// values, the transposed matrix, and the nonzero-split schedule used by the SpMM kernel.
//
// Section "Graph Neural Networks" of the paper defines the matrix (self-connections added,
// D^-1/2 (A+I) D^-1/2); section "Communication Schemes and their Analyses" keeps both A and A^T
// so that neither product needs a transposition (or, here, floating-point atomics) at run time.
//
// Entries are encoded as 64-bit keys row<<32|col; a radix sort of the keys followed by the
// removal of equal neighbours yields the canonical row-major order with ascending columns.  The
// device-wide sort, selection and prefix sum are the ones of prims.h.
#include <cstring>
#include <new>

#include "common.h"
#include "prims.h"
#include "build_util.h"

namespace gcn {

static constexpr uint64_t INVALID_KEY = ~0ull;

// ---- kernels ---------------------------------------------------------------------------------

__global__ void k_check_ids(int64_t m, int64_t n, const int32_t* __restrict__ src,
                            const int32_t* __restrict__ dst, int* __restrict__ bad) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= m) return;
    int32_t u = src[e], v = dst[e];
    if (u < 0 || v < 0 || u >= n || v >= n) *bad = 1;
}

// One key per stored direction of each input pair; pairs with u == v become INVALID_KEY, which
// sorts behind every real key.  Self loops are appended after the 'mult*m' edge keys.
__global__ void k_make_keys(int64_t m, int64_t n, const int32_t* __restrict__ src,
                            const int32_t* __restrict__ dst, int symmetrise, int self_loops,
                            uint64_t* __restrict__ keys) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int mult = symmetrise ? 2 : 1;
    if (t < m) {
        uint64_t u = (uint32_t)src[t], v = (uint32_t)dst[t];
        bool loop = (u == v);
        keys[t * mult] = loop ? INVALID_KEY : (u << 32 | v);
        if (symmetrise) keys[t * mult + 1] = loop ? INVALID_KEY : (v << 32 | u);
    } else if (self_loops && t < m + n) {
        uint64_t i = (uint64_t)(t - m);
        keys[m * mult + (t - m)] = i << 32 | i;
    }
}

__global__ void k_degrees(int64_t n, const int64_t* __restrict__ rowptr, int32_t* __restrict__ deg,
                          int32_t* __restrict__ max_deg, unsigned long long* __restrict__ n_nonempty) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int32_t d = 0;
    if (i < n) {
        d = (int32_t)(rowptr[i + 1] - rowptr[i]);
        if (deg) deg[i] = d;
    }
    // one integer atomic per wavefront instead of one per row
    int32_t m = d;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const int32_t o = __shfl_xor(m, s, 64);
        m = o > m ? o : m;
    }
    const unsigned long long nz = __popcll(__ballot(d > 0));
    if ((threadIdx.x & 63) == 0) {
        if (max_deg) atomicMax(max_deg, m);
        if (n_nonempty && nz) atomicAdd(n_nonempty, nz);
    }
}

// val(i,j) = (float)(1 / sqrt(d_i d_j)): exact integer product in double, correctly rounded
// square root and division, one rounding to float -- the same value on any IEEE machine.
// norm 2 is the row normalisation D^-1 (A+I): val(i,j) = (float)(1 / d_i).
__global__ void k_values(int64_t nnz, const uint64_t* __restrict__ keys, const int32_t* __restrict__ deg,
                         int norm, float* __restrict__ val) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    if (norm == 0) {
        val[k] = 1.0f;
        return;
    }
    uint64_t key = keys[k];
    double di = (double)deg[key >> 32], dj = (double)deg[key & 0xffffffffu];
    if (norm == 2) val[k] = (float)__ddiv_rn(1.0, di);
    else {
        // a vertex whose row is empty (no self loops, no outgoing edge) scales by 0: D^-1/2 as a pseudo-inverse,
        // the same convention as the per-vertex factors of the value-free product
        const double dd = __dmul_rn(di, dj);
        val[k] = dd > 0.0 ? (float)__ddiv_rn(1.0, __dsqrt_rn(dd)) : 0.f;
    }
}

__global__ void k_swap_halves(int64_t nnz, const uint64_t* __restrict__ keys, uint64_t* __restrict__ out) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < nnz) out[k] = (keys[k] << 32) | (keys[k] >> 32);
}

// keys row<<32|col from compressed rows: thread k finds its row by bisection on rowptr.
__global__ void k_keys_from_csr(int64_t nnz, int64_t n, const int64_t* __restrict__ rowptr,
                                const int32_t* __restrict__ colidx, uint64_t* __restrict__ keys) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    int64_t lo = 0, hi = n;   // largest r with rowptr[r] <= k
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= k) lo = mid; else hi = mid;
    }
    keys[k] = ((uint64_t)lo << 32) | (uint32_t)colidx[k];
}

__global__ void k_validate_rowptr(int64_t n, const int64_t* __restrict__ rowptr, int* __restrict__ bad) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (i == 0 && rowptr[0] != 0) *bad = 1;
    if (rowptr[i + 1] < rowptr[i]) *bad = 1;
}

// after k_keys_from_csr: keys must be strictly increasing and columns inside [0,n)
__global__ void k_validate_keys(int64_t nnz, int64_t n, const uint64_t* __restrict__ keys, int* __restrict__ bad) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    if ((keys[k] & 0xffffffffu) >= (uint64_t)n) *bad = 1;
    if (k > 0 && keys[k] <= keys[k - 1]) *bad = 1;
}

__global__ void k_fill_f32(int64_t count, float v, float* __restrict__ out) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < count) out[k] = v;
}

// ---- schedule kernels ---------------------------------------------------------------------------

struct NonEmpty {
    const int64_t* rowptr;
    __device__ bool operator()(const int32_t& r) const { return rowptr[r + 1] > rowptr[r]; }
};
struct IsEmpty {
    const int64_t* rowptr;
    __device__ bool operator()(const int32_t& r) const { return rowptr[r + 1] == rowptr[r]; }
};

__global__ void k_ne_rowptr(int64_t n_ne, int64_t nnz, const int32_t* __restrict__ ne_rows,
                            const int64_t* __restrict__ rowptr, int64_t* __restrict__ out) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n_ne) out[q] = rowptr[ne_rows[q]];
    if (q == n_ne) out[q] = nnz;
}

// ---- host helpers ---------------------------------------------------------------------------------

static int sort_keys(uint64_t* in, uint64_t* out, int64_t count, int64_t n, hipStream_t s) {
    unsigned end_bit = 64;   // INVALID_KEY uses every bit
    (void)n;
    return prims::sort_keys<uint64_t>(in, out, (size_t)count, end_bit, s);
}

// From sorted distinct keys (row<<32|col) fill rowptr/colidx of `m` (allocates them).
static int compress_keys(Matrix& m, int64_t n, int64_t nnz, const uint64_t* keys, hipStream_t s) {
    GCN_TRY(device_alloc_t(&m.rowptr, (size_t)n + 1));
    GCN_TRY(device_alloc_t(&m.colidx, (size_t)nnz));
    hipLaunchKernelGGL(k_compress, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, n, keys, m.rowptr, m.colidx);
    GCN_LAUNCH_CHECK();
    return GCN_OK;
}

// The chunks c >= 1 whose first entry continues a row begun earlier and that are the first such chunk
// of that row: exactly the chunks for which the fix-up kernel has work.
struct LeadsCarry {
    const uint32_t* flags;
    const int32_t* sub_row;
    const int64_t* rp;
    __device__ bool operator()(const int32_t& c0) const {
        const int64_t c = (int64_t)c0 + 1;
        const int64_t j0 = c * SUBS_PER_CHUNK;
        if (flags[j0] & 1u) return false;
        return c == rp[sub_row[j0]] / CHUNK + 1;
    }
};

__global__ void k_add_one(int64_t count, int32_t* __restrict__ v) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) v[t] += 1;
}

int build_fix_list(const uint32_t* flags, const int32_t* sub_row, const int64_t* rp, int64_t nchunks, int32_t** list,
                   int64_t* count, hipStream_t s) {
    *count = 0;
    if (nchunks <= 1) return GCN_OK;
    if (nchunks >= (1ll << 31)) { *count = -1; return GCN_OK; }          // keep the exhaustive form
    TempBuf sel;
    GCN_TRY(sel.alloc((size_t)(nchunks - 1) * 4));
    LeadsCarry pred{flags, sub_row, rp};
    int64_t nsel = 0;
    GCN_TRY(prims::select_indices(nchunks - 1, pred, sel.as<int32_t>(), &nsel, s));
    if (nsel > 0) {
        GCN_TRY(device_alloc_t(list, (size_t)nsel));
        GCN_HIP_TRY(hipMemcpyAsync(*list, sel.p, (size_t)nsel * 4, hipMemcpyDeviceToDevice, s));
        hipLaunchKernelGGL(k_add_one, dim3(blocks_for(nsel)), dim3(TPB), 0, s, nsel, *list);
        GCN_LAUNCH_CHECK();
        GCN_HIP_TRY(hipStreamSynchronize(s));
    }
    *count = nsel;
    return GCN_OK;
}

int build_schedule(Matrix& m, int64_t n, int64_t nnz, hipStream_t s) {
    m.nsub = (nnz + SUB - 1) / SUB;
    m.nchunks = (nnz + CHUNK - 1) / CHUNK;
    TempBuf counters;
    GCN_TRY(counters.alloc(16));
    GCN_HIP_TRY(hipMemsetAsync(counters.p, 0, 16, s));
    hipLaunchKernelGGL(k_degrees, dim3(blocks_for(n)), dim3(TPB), 0, s, n, m.rowptr, (int32_t*)nullptr,
                       (int32_t*)counters.p, (unsigned long long*)((char*)counters.p + 8));
    GCN_LAUNCH_CHECK();
    struct { int32_t maxd; int32_t pad; unsigned long long nne; } h;
    GCN_HIP_TRY(hipMemcpyAsync(&h, counters.p, 16, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    m.max_degree = h.maxd;
    m.n_ne = (int64_t)h.nne;
    const int64_t* rp = m.rowptr;
    if (m.n_ne < n) {
        GCN_TRY(device_alloc_t(&m.ne_rows, (size_t)m.n_ne));
        GCN_TRY(device_alloc_t(&m.ne_rowptr, (size_t)m.n_ne + 1));
        NonEmpty pred{m.rowptr};
        GCN_TRY(prims::select_indices(n, pred, m.ne_rows, nullptr, s));
        hipLaunchKernelGGL(k_ne_rowptr, dim3(blocks_for(m.n_ne + 1)), dim3(TPB), 0, s, m.n_ne, nnz, m.ne_rows,
                           m.rowptr, m.ne_rowptr);
        GCN_LAUNCH_CHECK();
        GCN_TRY(device_alloc_t(&m.empty_rows, (size_t)(n - m.n_ne)));
        IsEmpty epred{m.rowptr};
        GCN_TRY(prims::select_indices(n, epred, m.empty_rows, nullptr, s));
        GCN_HIP_TRY(hipStreamSynchronize(s));
        rp = m.ne_rowptr;
    }
    GCN_TRY(device_alloc_t(&m.flags, (size_t)m.nsub + SUBS_PER_CHUNK));   // padded: one chunk of zero words
    GCN_TRY(device_alloc_t(&m.sub_row, (size_t)m.nsub + SUBS_PER_CHUNK));
    GCN_HIP_TRY(hipMemsetAsync(m.flags, 0, ((size_t)m.nsub + SUBS_PER_CHUNK) * sizeof(uint32_t), s));
    GCN_HIP_TRY(hipMemsetAsync(m.sub_row, 0, ((size_t)m.nsub + SUBS_PER_CHUNK) * sizeof(int32_t), s));
    if (nnz > 0) {
        hipLaunchKernelGGL(k_row_flags, dim3(blocks_for(m.n_ne)), dim3(TPB), 0, s, m.n_ne, rp, m.flags);
        GCN_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_sub_rows, dim3(blocks_for(m.nsub)), dim3(TPB), 0, s, m.nsub, m.n_ne, rp, m.sub_row);
        GCN_LAUNCH_CHECK();
    }
    GCN_HIP_TRY(hipStreamSynchronize(s));
    if (nnz > 0) GCN_TRY(build_fix_list(m.flags, m.sub_row, rp, m.nchunks, &m.fix_list, &m.n_fix, s));
    return GCN_OK;
}

// A^T of `a` from A's sorted keys and values: swap key halves, stable radix sort with the values
// as payload.  Within a column the rows keep their ascending order.
static int build_transpose(gcn_csr* a, const uint64_t* keys, uint64_t* scratch_keys, hipStream_t s) {
    const int64_t nnz = a->nnz, n = a->ncols;            // A^T has ncols rows
    TempBuf kin, vtmp;
    GCN_TRY(kin.alloc((size_t)nnz * 8));
    GCN_TRY(device_alloc_t(&a->At.val, (size_t)nnz));
    hipLaunchKernelGGL(k_swap_halves, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, keys, kin.as<uint64_t>());
    GCN_LAUNCH_CHECK();
    unsigned end_bit = 32 + bits_for(n);                 // low half: rows of A, high half: its columns
    GCN_TRY((prims::sort_pairs<uint64_t, float>(kin.as<uint64_t>(), scratch_keys, a->A.val, a->At.val, (size_t)nnz,
                                                end_bit, s)));
    a->At.nrows = n;
    a->At.ncols = a->n;
    GCN_TRY(compress_keys(a->At, n, nnz, scratch_keys, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    GCN_TRY(build_schedule(a->At, n, nnz, s));
    a->has_t = true;
    return GCN_OK;
}

static int create_impl(gcn_csr* a, int64_t n, int64_t m, const int32_t* src, const int32_t* dst, uint32_t flags,
                       hipStream_t s) {
    const bool sym = flags & GCN_SYMMETRISE, loops = flags & GCN_ADD_SELF_LOOPS;
    const int mult = sym ? 2 : 1;
    const int64_t cap = m * mult + (loops ? n : 0);

    TempBuf bad;
    GCN_TRY(bad.alloc(sizeof(int)));
    GCN_HIP_TRY(hipMemsetAsync(bad.p, 0, sizeof(int), s));
    if (m > 0) {
        hipLaunchKernelGGL(k_check_ids, dim3(blocks_for(m)), dim3(TPB), 0, s, m, n, src, dst, bad.as<int>());
        GCN_LAUNCH_CHECK();
    }
    int hbad = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&hbad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    if (hbad) return fail(GCN_ERR_RANGE, "gcn_csr_create: a vertex id is outside [0, %lld)", (long long)n);

    TempBuf k0, k1;
    GCN_TRY(k0.alloc((size_t)cap * 8));
    GCN_TRY(k1.alloc((size_t)cap * 8));
    int64_t nnz = 0;
    if (cap > 0) {
        hipLaunchKernelGGL(k_make_keys, dim3(blocks_for(m + (loops ? n : 0))), dim3(TPB), 0, s, m, n, src, dst,
                           (int)sym, (int)loops, k0.as<uint64_t>());
        GCN_LAUNCH_CHECK();
        GCN_TRY(sort_keys(k0.as<uint64_t>(), k1.as<uint64_t>(), cap, n, s));
        int64_t hcnt = 0;
        uint64_t last = 0;
        GCN_TRY(prims::unique_keys(k1.as<uint64_t>(), k0.as<uint64_t>(), cap, &hcnt, s));
        if (hcnt > 0) {
            GCN_HIP_TRY(hipMemcpyAsync(&last, k0.as<uint64_t>() + (hcnt - 1), 8, hipMemcpyDeviceToHost, s));
            GCN_HIP_TRY(hipStreamSynchronize(s));
            if (last == INVALID_KEY) hcnt -= 1;
        }
        nnz = hcnt;
    }
    const uint64_t* keys = k0.as<uint64_t>();   // sorted, distinct, nnz of them
    a->n = n;
    a->ncols = n;
    a->nnz = nnz;
    a->A.nrows = a->A.ncols = n;
    GCN_TRY(compress_keys(a->A, n, nnz, keys, s));
    GCN_TRY(device_alloc_t(&a->deg, (size_t)n));
    GCN_TRY(device_alloc_t(&a->A.val, (size_t)nnz));
    hipLaunchKernelGGL(k_degrees, dim3(blocks_for(n)), dim3(TPB), 0, s, n, a->A.rowptr, a->deg, (int32_t*)nullptr,
                       (unsigned long long*)nullptr);
    GCN_LAUNCH_CHECK();
    if (nnz > 0) {
        hipLaunchKernelGGL(k_values, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, keys, a->deg,
                           (flags & GCN_NORM_ROW) ? 2 : ((flags & GCN_NORM_SYM) ? 1 : 0), a->A.val);
        GCN_LAUNCH_CHECK();
    }
    if ((flags & GCN_NORM_SYM) && n > 0) {
        GCN_TRY(device_alloc_t(&a->inv_sqrt_deg, (size_t)n));
        GCN_TRY(inv_sqrt_deg_launch(n, a->deg, a->inv_sqrt_deg, s));
    }
    GCN_HIP_TRY(hipStreamSynchronize(s));
    GCN_TRY(build_schedule(a->A, n, nnz, s));
    if (flags & GCN_BUILD_TRANSPOSE) GCN_TRY(build_transpose(a, keys, k1.as<uint64_t>(), s));
    return GCN_OK;
}

static int from_csr_impl(gcn_csr* a, int64_t n, int64_t ncols, const int64_t* rowptr, const int32_t* colidx,
                         const float* val, uint32_t flags, hipStream_t s) {
    TempBuf bad;
    GCN_TRY(bad.alloc(sizeof(int)));
    GCN_HIP_TRY(hipMemsetAsync(bad.p, 0, sizeof(int), s));
    hipLaunchKernelGGL(k_validate_rowptr, dim3(blocks_for(n)), dim3(TPB), 0, s, n, rowptr, bad.as<int>());
    GCN_LAUNCH_CHECK();
    int hbad = 0;
    int64_t nnz = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&hbad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipMemcpyAsync(&nnz, rowptr + n, 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    if (hbad || nnz < 0) return fail(GCN_ERR_UNSORTED, "gcn_csr_create_from_csr: rowptr must start at 0 and not decrease");
    if (nnz > 0 && !colidx) return fail(GCN_ERR_BADARG, "gcn_csr_create_from_csr: NULL colidx");
    a->n = n;
    a->ncols = ncols;
    a->nnz = nnz;
    a->A.nrows = n;
    a->A.ncols = ncols;
    GCN_TRY(device_alloc_t(&a->A.rowptr, (size_t)n + 1));
    GCN_TRY(device_alloc_t(&a->A.colidx, (size_t)nnz));
    GCN_TRY(device_alloc_t(&a->A.val, (size_t)nnz));
    GCN_TRY(device_alloc_t(&a->deg, (size_t)n));
    GCN_HIP_TRY(hipMemcpyAsync(a->A.rowptr, rowptr, ((size_t)n + 1) * 8, hipMemcpyDeviceToDevice, s));
    TempBuf keys, k1;
    GCN_TRY(keys.alloc((size_t)nnz * 8));
    if (nnz > 0) {
        GCN_HIP_TRY(hipMemcpyAsync(a->A.colidx, colidx, (size_t)nnz * 4, hipMemcpyDeviceToDevice, s));
        if (val) GCN_HIP_TRY(hipMemcpyAsync(a->A.val, val, (size_t)nnz * 4, hipMemcpyDeviceToDevice, s));
        else {
            hipLaunchKernelGGL(k_fill_f32, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, 1.0f, a->A.val);
            GCN_LAUNCH_CHECK();
        }
        hipLaunchKernelGGL(k_keys_from_csr, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, n, a->A.rowptr, a->A.colidx,
                           keys.as<uint64_t>());
        GCN_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_validate_keys, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, ncols, keys.as<uint64_t>(),
                           bad.as<int>());
        GCN_LAUNCH_CHECK();
        GCN_HIP_TRY(hipMemcpyAsync(&hbad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
        GCN_HIP_TRY(hipStreamSynchronize(s));
        if (hbad) return fail(GCN_ERR_UNSORTED, "gcn_csr_create_from_csr: columns must be strictly ascending per row and inside [0,n)");
    }
    hipLaunchKernelGGL(k_degrees, dim3(blocks_for(n)), dim3(TPB), 0, s, n, a->A.rowptr, a->deg, (int32_t*)nullptr,
                       (unsigned long long*)nullptr);
    GCN_LAUNCH_CHECK();
    GCN_HIP_TRY(hipStreamSynchronize(s));
    GCN_TRY(build_schedule(a->A, n, nnz, s));
    if (flags & GCN_BUILD_TRANSPOSE) {
        GCN_TRY(k1.alloc((size_t)nnz * 8));
        GCN_TRY(build_transpose(a, keys.as<uint64_t>(), k1.as<uint64_t>(), s));
    }
    return GCN_OK;
}

}  // namespace gcn

using namespace gcn;

namespace {
struct Pay4 { uint32_t a; };
struct Pay8 { uint32_t a, b; };
struct Pay12 { uint32_t a, b, c; };

template <typename K>
int radix_sort_by_payload(int64_t n, const void* kin, void* kout, int payload_bytes, const void* pin, void* pout,
                          unsigned end_bit, bool desc, hipStream_t s) {
    using namespace gcn::prims;
    const K* ki = (const K*)kin;
    K* ko = (K*)kout;
    switch (payload_bytes) {
        case 0: return radix_sort<K, NoValue>(ki, ko, (const NoValue*)nullptr, (NoValue*)nullptr, (size_t)n, end_bit, desc, s);
        case 4: return radix_sort<K, Pay4>(ki, ko, (const Pay4*)pin, (Pay4*)pout, (size_t)n, end_bit, desc, s);
        case 8: return radix_sort<K, Pay8>(ki, ko, (const Pay8*)pin, (Pay8*)pout, (size_t)n, end_bit, desc, s);
        case 12: return radix_sort<K, Pay12>(ki, ko, (const Pay12*)pin, (Pay12*)pout, (size_t)n, end_bit, desc, s);
        default: return gcn::fail(GCN_ERR_BADARG, "gcn_radix_sort: payload_bytes must be 0, 4, 8 or 12");
    }
}
}  // namespace

extern "C" {

int gcn_csr_create(gcn_csr** out, int64_t n, int64_t n_edges, const int32_t* src, const int32_t* dst,
                   uint32_t flags, void* stream) {
    if (!out) return fail(GCN_ERR_BADARG, "gcn_csr_create: NULL out");
    *out = nullptr;
    if (n <= 0 || n_edges < 0) return fail(GCN_ERR_BADARG, "gcn_csr_create: n must be positive and n_edges non-negative");
    if (n >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_csr_create: n must be below 2^31");
    if (n_edges > 0 && (!src || !dst)) return fail(GCN_ERR_BADARG, "gcn_csr_create: NULL edge arrays");
    if (n_edges > (1ll << 40)) return fail(GCN_ERR_RANGE, "gcn_csr_create: too many edges");
    if ((flags & GCN_NORM_SYM) && (flags & GCN_NORM_ROW)) return fail(GCN_ERR_BADARG, "gcn_csr_create: choose one normalisation");
    gcn_csr* a = new (std::nothrow) gcn_csr();
    if (!a) return fail(GCN_ERR_OOM, "host allocation failed");
    (void)hipGetDevice(&a->device);
    int rc = create_impl(a, n, n_edges, src, dst, flags, (hipStream_t)stream);
    if (rc != GCN_OK) {
        gcn_csr_destroy(a);
        return rc;
    }
    *out = a;
    return GCN_OK;
}

int gcn_csr_create_from_csr(gcn_csr** out, int64_t n, const int64_t* rowptr, const int32_t* colidx,
                            const float* val, uint32_t flags, void* stream) {
    if (!out) return fail(GCN_ERR_BADARG, "gcn_csr_create_from_csr: NULL out");
    *out = nullptr;
    if (n <= 0 || !rowptr) return fail(GCN_ERR_BADARG, "gcn_csr_create_from_csr: n must be positive, rowptr non-NULL");
    if (n >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_csr_create_from_csr: n must be below 2^31");
    gcn_csr* a = new (std::nothrow) gcn_csr();
    if (!a) return fail(GCN_ERR_OOM, "host allocation failed");
    (void)hipGetDevice(&a->device);
    int rc = from_csr_impl(a, n, n, rowptr, colidx, val, flags, (hipStream_t)stream);
    if (rc != GCN_OK) {
        gcn_csr_destroy(a);
        return rc;
    }
    *out = a;
    return GCN_OK;
}

int gcn_csr_create_from_csr_rect(gcn_csr** out, int64_t n_rows, int64_t n_cols, const int64_t* rowptr,
                                 const int32_t* colidx, const float* val, uint32_t flags, void* stream) {
    if (!out) return fail(GCN_ERR_BADARG, "gcn_csr_create_from_csr_rect: NULL out");
    *out = nullptr;
    if (n_rows <= 0 || n_cols <= 0 || !rowptr) return fail(GCN_ERR_BADARG, "gcn_csr_create_from_csr_rect: sizes must be positive, rowptr non-NULL");
    if (n_rows >= (1ll << 31) || n_cols >= (1ll << 31)) return fail(GCN_ERR_RANGE, "gcn_csr_create_from_csr_rect: sizes must be below 2^31");
    gcn_csr* a = new (std::nothrow) gcn_csr();
    if (!a) return fail(GCN_ERR_OOM, "host allocation failed");
    (void)hipGetDevice(&a->device);
    int rc = from_csr_impl(a, n_rows, n_cols, rowptr, colidx, val, flags, (hipStream_t)stream);
    if (rc != GCN_OK) {
        gcn_csr_destroy(a);
        return rc;
    }
    *out = a;
    return GCN_OK;
}

int gcn_radix_sort(int64_t n, int key_bytes, const void* keys_in, void* keys_out, int payload_bytes,
                   const void* payload_in, void* payload_out, int end_bit, int descending, void* stream) {
    using gcn::fail;
    if (n < 0 || end_bit < 0) return fail(GCN_ERR_BADARG, "gcn_radix_sort: negative size");
    if (n == 0) return GCN_OK;
    if (!keys_in || !keys_out || keys_in == keys_out) return fail(GCN_ERR_BADARG, "gcn_radix_sort: keys NULL or in place");
    if (payload_bytes != 0 && (!payload_in || !payload_out || payload_in == payload_out))
        return fail(GCN_ERR_BADARG, "gcn_radix_sort: payload NULL or in place");
    if (key_bytes == 8)
        return radix_sort_by_payload<uint64_t>(n, keys_in, keys_out, payload_bytes, payload_in, payload_out,
                                               (unsigned)end_bit, descending != 0, (hipStream_t)stream);
    if (key_bytes == 4)
        return radix_sort_by_payload<uint32_t>(n, keys_in, keys_out, payload_bytes, payload_in, payload_out,
                                               (unsigned)end_bit, descending != 0, (hipStream_t)stream);
    return fail(GCN_ERR_BADARG, "gcn_radix_sort: key_bytes must be 4 or 8");
}

int gcn_exclusive_scan_i64(int64_t n, const int64_t* in, int64_t* out, void* stream) {
    if (n < 0) return gcn::fail(GCN_ERR_BADARG, "gcn_exclusive_scan_i64: negative size");
    if (n == 0) return GCN_OK;
    if (!in || !out) return gcn::fail(GCN_ERR_BADARG, "gcn_exclusive_scan_i64: NULL pointer");
    return gcn::prims::exclusive_scan<int64_t>(in, out, (size_t)n, (hipStream_t)stream);
}

int gcn_unique_u64(int64_t n, const uint64_t* keys_in, uint64_t* keys_out, int64_t* count, void* stream) {
    if (n < 0 || !count) return gcn::fail(GCN_ERR_BADARG, "gcn_unique_u64: negative size or NULL count");
    *count = 0;
    if (n == 0) return GCN_OK;
    if (!keys_in || !keys_out || keys_in == keys_out) return gcn::fail(GCN_ERR_BADARG, "gcn_unique_u64: keys NULL or in place");
    return gcn::prims::unique_keys(keys_in, keys_out, n, count, (hipStream_t)stream);
}

}  // extern "C"
