// Small host-side helpers shared by the graph-construction sources.
#pragma once
#include "common.h"

namespace gcn {

static constexpr int TPB = 256;

static inline unsigned blocks_for(int64_t work, int per_block = TPB) {
    int64_t b = (work + per_block - 1) / per_block;
    return (unsigned)(b < 1 ? 1 : b);
}

struct TempBuf {   // frees on scope exit
    void* p = nullptr;
    ~TempBuf() { device_free(p); }
    int alloc(size_t bytes) { device_free(p); return device_alloc(&p, bytes); }
    template <typename T> T* as() const { return (T*)p; }
};

// Bits needed for the values 0 .. n-1 (at least 1, at most 32).
static inline unsigned bits_for(int64_t n) {
    unsigned b = 1;
    while (b < 32 && (1ll << b) < n) ++b;
    return b;
}

// ---- kernels used by more than one construction source (one copy per source file) ----

// Sorted distinct keys -> colidx and rowptr.  Entry k is the first of every row in
// (row(k-1), row(k)], so its thread writes rowptr for those rows; the last entry's thread also
// closes all rows behind it.
static __global__ void k_compress(int64_t nnz, int64_t n, const uint64_t* __restrict__ keys,
                           int64_t* __restrict__ rowptr, int32_t* __restrict__ colidx) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (nnz == 0) {
        for (int64_t r = k; r <= n; r += (int64_t)gridDim.x * blockDim.x) rowptr[r] = 0;
        return;
    }
    if (k >= nnz) return;
    uint64_t key = keys[k];
    int64_t r = (int64_t)(key >> 32);
    int64_t rp = k > 0 ? (int64_t)(keys[k - 1] >> 32) : -1;
    colidx[k] = (int32_t)(key & 0xffffffffu);
    for (int64_t q = rp + 1; q <= r; ++q) rowptr[q] = k;
    if (k == nnz - 1)
        for (int64_t q = r + 1; q <= n; ++q) rowptr[q] = nnz;
}

// One flag bit per stored entry that starts a (non-empty) row.
static __global__ void k_row_flags(int64_t n_ne, const int64_t* __restrict__ rp, uint32_t* __restrict__ flags) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_ne) return;
    int64_t k = rp[q];
    atomicOr(&flags[k >> 5], 1u << (k & 31));
}

// For every group of SUB entries, the (non-empty) row that its first entry belongs to, by bisection.
static __global__ void k_sub_rows(int64_t nsub, int64_t n_ne, const int64_t* __restrict__ rp, int32_t* __restrict__ sub_row) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= nsub) return;
    int64_t k = j * SUB, lo = 0, hi = n_ne;   // largest q with rp[q] <= k  (rp[0] == 0)
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (rp[mid] <= k) lo = mid; else hi = mid;
    }
    sub_row[j] = (int32_t)lo;
}

}  // namespace gcn
