// Alternative stored orders of a matrix for the SpMM kernels, built on first use from its compressed
// rows: the column-blocked copy (entries grouped by block of columns so that the gathered rows of the
// dense operand stay in L2), the sweep copy (tasks of rows whose entries are walked in column order
// with the accumulators in LDS) and the hub copy (long rows x most-used columns over a packed operand,
// the rest as a matrix of its own).  All of them hold the same entries as the matrix they come from;
// section "Graph Neural Networks" of the paper defines that matrix.
#include <new>

#include "common.h"
#include "prims.h"
#include "build_util.h"

namespace gcn {

// ---- column-blocked copy -----------------------------------------------------------------------------

// key = block<<32 | row, payload = col<<32 | value bits; thread k finds its row by bisection.
__global__ void k_block_keys(int64_t nnz, int64_t n, const int64_t* __restrict__ rowptr,
                             const int32_t* __restrict__ colidx, const float* __restrict__ val, int64_t cpb,
                             uint64_t* __restrict__ keys, uint64_t* __restrict__ payload) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= k) lo = mid; else hi = mid;
    }
    const uint32_t col = (uint32_t)colidx[k];
    keys[k] = ((uint64_t)(col / cpb) << 32) | (uint64_t)lo;
    payload[k] = ((uint64_t)col << 32) | (uint64_t)__float_as_uint(val[k]);
}

// Flag word j: bit b set iff sorted entry 32j+b opens a new (block,row) run; cnt[j] = set bits.
__global__ void k_block_flags(int64_t nnz, int64_t nsub, const uint64_t* __restrict__ keys,
                              uint32_t* __restrict__ flags, int32_t* __restrict__ cnt) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= nsub) return;
    uint32_t w = 0;
    const int64_t k0 = j * SUB;
    uint64_t prev = k0 > 0 ? keys[k0 - 1] : ~0ull;
    for (int b = 0; b < SUB && k0 + b < nnz; ++b) {
        const uint64_t cur = keys[k0 + b];
        if (k0 + b == 0 || cur != prev) w |= 1u << b;
        prev = cur;
    }
    flags[j] = w;
    cnt[j] = __popc(w);
}

// From the flags and their exclusive prefix counts: sub_row, the first entry rp[q] of every partial
// row q, and the sort key (row<<32 | q) that groups partial rows by the row they belong to.
__global__ void k_block_rows(int64_t /*nnz*/, int64_t nsub, const uint32_t* __restrict__ flags,
                             const int32_t* __restrict__ pre, const uint64_t* __restrict__ keys,
                             int32_t* __restrict__ sub_row, int64_t* __restrict__ rp, uint64_t* __restrict__ rowq) {
    int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= nsub) return;
    uint32_t w = flags[j];
    int32_t q = pre[j];
    sub_row[j] = q + (int32_t)(w & 1u) - 1;
    while (w) {
        const int b = __ffs(w) - 1;
        w &= w - 1;
        const int64_t k = j * SUB + b;
        rp[q] = k;
        rowq[q] = ((keys[k] & 0xffffffffull) << 32) | (uint64_t)(uint32_t)q;
        ++q;
    }
}

__global__ void k_block_unpack(int64_t nnz, const uint64_t* __restrict__ payload, int32_t* __restrict__ colidx,
                               float* __restrict__ val) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    colidx[k] = (int32_t)(payload[k] >> 32);
    val[k] = __uint_as_float((uint32_t)(payload[k] & 0xffffffffu));
}

__global__ void k_set_i64(int64_t* p, int64_t v) { *p = v; }

void free_blocked(Blocked& b);

int build_blocked(Matrix& m, int64_t nnz, int64_t cpb, hipStream_t s) {
    count_build();
    free_blocked(m.blk);
    Blocked& b = m.blk;
    if (nnz <= 0 || cpb <= 0) return fail(GCN_ERR_BADARG, "build_blocked: empty matrix or bad block width");
    const int64_t n = m.nrows;
    const int64_t nblocks = (m.ncols + cpb - 1) / cpb;
    const int64_t nsub = m.nsub;
    TempBuf k0, k1, p0, p1, cnt, pre;
    GCN_TRY(k0.alloc((size_t)nnz * 8));
    GCN_TRY(k1.alloc((size_t)nnz * 8));
    GCN_TRY(p0.alloc((size_t)nnz * 8));
    GCN_TRY(p1.alloc((size_t)nnz * 8));
    hipLaunchKernelGGL(k_block_keys, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, n, m.rowptr, m.colidx, m.val, cpb,
                       k0.as<uint64_t>(), p0.as<uint64_t>());
    GCN_LAUNCH_CHECK();
    const unsigned end_bit = 32 + bits_for(nblocks + 1);
    GCN_TRY((prims::sort_pairs<uint64_t, uint64_t>(k0.as<uint64_t>(), k1.as<uint64_t>(), p0.as<uint64_t>(),
                                                   p1.as<uint64_t>(), (size_t)nnz, end_bit, s)));
    k0.alloc(16);                                        // release the unsorted copies early
    p0.alloc(16);

    const size_t padded = (size_t)nsub + SUBS_PER_CHUNK;
    GCN_TRY(device_alloc_t(&b.flags, padded));
    GCN_TRY(device_alloc_t(&b.sub_row, padded));
    GCN_HIP_TRY(hipMemsetAsync(b.flags, 0, padded * sizeof(uint32_t), s));
    GCN_HIP_TRY(hipMemsetAsync(b.sub_row, 0, padded * sizeof(int32_t), s));
    GCN_TRY(cnt.alloc((size_t)nsub * 4));
    GCN_TRY(pre.alloc((size_t)nsub * 4));
    hipLaunchKernelGGL(k_block_flags, dim3(blocks_for(nsub)), dim3(TPB), 0, s, nnz, nsub, k1.as<uint64_t>(), b.flags,
                       cnt.as<int32_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY(prims::exclusive_scan<int32_t>(cnt.as<int32_t>(), pre.as<int32_t>(), (size_t)nsub, s));
    int32_t last_pre = 0, last_cnt = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&last_pre, pre.as<int32_t>() + (nsub - 1), 4, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipMemcpyAsync(&last_cnt, cnt.as<int32_t>() + (nsub - 1), 4, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    const int64_t R = (int64_t)last_pre + last_cnt;
    if (R <= 0) return fail(GCN_ERR_RANGE, "build_blocked: too many partial rows");   // int32 prefix overflowed

    GCN_TRY(device_alloc_t(&b.rp, (size_t)R + 1));
    TempBuf rq0, rq1;
    GCN_TRY(rq0.alloc((size_t)R * 8));
    GCN_TRY(rq1.alloc((size_t)R * 8));
    hipLaunchKernelGGL(k_block_rows, dim3(blocks_for(nsub)), dim3(TPB), 0, s, nnz, nsub, b.flags, pre.as<int32_t>(),
                       k1.as<uint64_t>(), b.sub_row, b.rp, rq0.as<uint64_t>());
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_set_i64, dim3(1), dim3(1), 0, s, b.rp + R, nnz);
    GCN_LAUNCH_CHECK();
    GCN_TRY(device_alloc_t(&b.colidx, (size_t)nnz));
    GCN_TRY(device_alloc_t(&b.val, (size_t)nnz));
    hipLaunchKernelGGL(k_block_unpack, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, p1.as<uint64_t>(), b.colidx, b.val);
    GCN_LAUNCH_CHECK();
    // group the partial rows by the row they belong to; inside a row q ascends, i.e. block order
    const unsigned end_bit2 = 32 + bits_for(n);
    GCN_TRY(prims::sort_keys<uint64_t>(rq0.as<uint64_t>(), rq1.as<uint64_t>(), (size_t)R, end_bit2, s));
    GCN_TRY(device_alloc_t(&b.rq_ptr, (size_t)n + 1));
    GCN_TRY(device_alloc_t(&b.rq_idx, (size_t)R));
    hipLaunchKernelGGL(k_compress, dim3(blocks_for(R)), dim3(TPB), 0, s, R, n, rq1.as<uint64_t>(), b.rq_ptr, b.rq_idx);
    GCN_LAUNCH_CHECK();
    GCN_HIP_TRY(hipStreamSynchronize(s));
    b.cols_per_block = cpb;
    b.nblocks = (int32_t)nblocks;
    b.nrows = R;
    GCN_TRY(build_fix_list(b.flags, b.sub_row, b.rp, (nnz + CHUNK - 1) / CHUNK, &b.fix_list, &b.n_fix, s));
    return GCN_OK;
}

// ---- sweep copy -----------------------------------------------------------------------------------------

struct SweepPayload { int32_t col; float val; int32_t row; };

// One thread per task walks the task's entries in ascending column order and packs them into steps
// of `groups` entries whose rows are all different (the lane groups of a step then add to different
// rows in LDS).  An entry whose row is already in the step waits in a short list and opens one of the
// next steps, so the stored order stays within a few steps of the column order.  With out == NULL
// only the number of steps is counted (task_len, sort_key, padded_len); otherwise the entries are
// written to task_base[t] + step*groups + slot.
__global__ void k_sweep_pack(int64_t ntasks, int32_t rb, int32_t groups, const int64_t* __restrict__ task_ptr,
                             const SweepPayload* __restrict__ payload, const int64_t* __restrict__ task_base,
                             int32_t* __restrict__ colidx, float* __restrict__ val, uint8_t* __restrict__ lrow,
                             int32_t* __restrict__ task_len, uint32_t* __restrict__ sort_key,
                             int64_t* __restrict__ padded_len) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ntasks) return;
    constexpr int D = 24;                       // entries that may wait at one time
    const int64_t lo = task_ptr[t], hi = task_ptr[t + 1];
    const int64_t base = task_base ? task_base[t] : 0;
    int64_t wait[D];
    int nw = 0;
    int64_t i = lo, step = 0;
    while (i < hi || nw > 0) {
        uint64_t m0 = 0, m1 = 0, m2 = 0, m3 = 0;                    // rows (0..255) present in this step
        int cnt = 0;
        auto taken = [&](int r) {
            const uint64_t bit = 1ull << (r & 63);
            const int q = r >> 6;
            return ((q == 0 ? m0 : q == 1 ? m1 : q == 2 ? m2 : m3) & bit) != 0;
        };
        auto take = [&](int r) {
            const uint64_t bit = 1ull << (r & 63);
            const int q = r >> 6;
            if (q == 0) m0 |= bit; else if (q == 1) m1 |= bit; else if (q == 2) m2 |= bit; else m3 |= bit;
        };
        auto emit = [&](int64_t pos, int r) {
            if (colidx) {
                const SweepPayload pl = payload[pos];
                const int64_t dst = base + step * groups + cnt;
                colidx[dst] = pl.col;
                val[dst] = pl.val;
                lrow[dst] = (uint8_t)r;
            }
            ++cnt;
        };
        int keep = 0;
        for (int d = 0; d < nw; ++d) {                              // waiting entries first, oldest first
            const int64_t pos = wait[d];
            const int r = payload[pos].row % rb;
            if (cnt < groups && !taken(r)) { take(r); emit(pos, r); }
            else wait[keep++] = pos;
        }
        nw = keep;
        while (cnt < groups && i < hi) {
            const int r = payload[i].row % rb;
            if (taken(r)) {
                if (nw == D) break;                                 // close the step short rather than reorder further
                wait[nw++] = i++;
            } else {
                take(r);
                emit(i++, r);
            }
        }
        ++step;                                                     // every step places at least one entry
    }
    if (!colidx) {
        const int64_t len = step * groups;
        task_len[t] = (int32_t)len;
        sort_key[t] = (uint32_t)len;
        padded_len[t] = (len + 15) & ~15ll;
    }
}

// key = task | column for entries of light rows, one bit above that for entries of heavy rows (they
// sort behind everything and keep their (row, col) order: the sort is stable).
__global__ void k_sweep_keys(int64_t nnz, int64_t n, const int64_t* __restrict__ rowptr,
                             const int32_t* __restrict__ colidx, const float* __restrict__ val, int32_t rb,
                             int32_t heavy_th, unsigned cbits, uint64_t heavy_key,
                             uint64_t* __restrict__ keys, SweepPayload* __restrict__ payload) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= k) lo = mid; else hi = mid;
    }
    const int32_t col = colidx[k];
    const bool heavy = rowptr[lo + 1] - rowptr[lo] > heavy_th;
    keys[k] = heavy ? heavy_key
                    : ((uint64_t)(lo / rb) << cbits) | (uint64_t)(uint32_t)col;
    payload[k] = SweepPayload{col, val[k], (int32_t)lo};
}

// seg_ptr[t] = first sorted position of task t; seg_ptr[ntasks] = number of light entries
__global__ void k_sweep_seg_ptr(int64_t nseg, int64_t nnz, unsigned cbits, uint64_t heavy_key,
                                const uint64_t* __restrict__ keys, int64_t* __restrict__ seg_ptr) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q > nseg) return;
    const uint64_t want = q == nseg ? heavy_key : ((uint64_t)q << cbits);
    int64_t lo = 0, hi = nnz;      // first position with keys[pos] >= want
    while (lo < hi) {
        int64_t mid = (lo + hi) >> 1;
        if (keys[mid] < want) lo = mid + 1; else hi = mid;
    }
    seg_ptr[q] = lo;
}

__global__ void k_iota_i32(int64_t count, int32_t* __restrict__ out) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) out[t] = (int32_t)t;
}

// Heavy rows: sorted position first + k goes to position k of their own arrays.
__global__ void k_sweep_unpack(int64_t count, int64_t first, const SweepPayload* __restrict__ payload,
                               int32_t* __restrict__ colidx, float* __restrict__ val) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const SweepPayload p = payload[first + k];
    colidx[k] = p.col;
    val[k] = p.val;
}

struct HeavyRow {
    const int64_t* rowptr;
    int32_t th;
    __device__ bool operator()(const int32_t& r) const { return rowptr[r + 1] - rowptr[r] > th; }
};

__global__ void k_heavy_len(int64_t nh, const int32_t* __restrict__ rows, const int64_t* __restrict__ rowptr,
                            int64_t* __restrict__ len) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nh) len[q] = rowptr[rows[q] + 1] - rowptr[rows[q]];
    if (q == nh) len[q] = 0;
}

int build_sweep(Matrix& m, int64_t nnz, int32_t groups, int32_t rb, int32_t heavy_th, hipStream_t s) {
    count_build();
    free_sweep(m.swp);
    Sweep& w = m.swp;
    if (nnz <= 0 || rb <= 0 || rb > 256 || (groups != 8 && groups != 16))
        return fail(GCN_ERR_BADARG, "build_sweep: bad parameters");
    const int64_t n = m.nrows;
    const int64_t ntasks = (n + rb - 1) / rb;
    const unsigned cbits = bits_for(m.ncols);
    const unsigned tbits = bits_for(ntasks + 1);
    if (cbits + tbits + 1 > 63) return fail(GCN_ERR_RANGE, "build_sweep: key does not fit");
    const uint64_t heavy_key = 1ull << (cbits + tbits);

    // entries sorted by (task, column); heavy rows behind them in (row, column) order
    TempBuf k0, k1, p0, p1, seg;
    GCN_TRY(k0.alloc((size_t)nnz * 8));
    GCN_TRY(k1.alloc((size_t)nnz * 8));
    GCN_TRY(p0.alloc((size_t)nnz * sizeof(SweepPayload)));
    GCN_TRY(p1.alloc((size_t)nnz * sizeof(SweepPayload)));
    hipLaunchKernelGGL(k_sweep_keys, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, n, m.rowptr, m.colidx, m.val, rb, heavy_th,
                       cbits, heavy_key, k0.as<uint64_t>(), p0.as<SweepPayload>());
    GCN_LAUNCH_CHECK();
    const unsigned end_bit = cbits + tbits + 1;
    GCN_TRY((prims::sort_pairs<uint64_t, SweepPayload>(k0.as<uint64_t>(), k1.as<uint64_t>(), p0.as<SweepPayload>(),
                                                       p1.as<SweepPayload>(), (size_t)nnz, end_bit, s)));
    k0.alloc(16);
    p0.alloc(16);
    GCN_TRY(seg.alloc(((size_t)ntasks + 1) * 8));
    hipLaunchKernelGGL(k_sweep_seg_ptr, dim3(blocks_for(ntasks + 1)), dim3(TPB), 0, s, ntasks, nnz, cbits, heavy_key,
                       k1.as<uint64_t>(), seg.as<int64_t>());
    GCN_LAUNCH_CHECK();
    k1.alloc(16);

    // pass 1: steps per task; then the longest-first order and the offsets of the tasks
    GCN_TRY(device_alloc_t(&w.task_base, (size_t)ntasks));
    GCN_TRY(device_alloc_t(&w.task_len, (size_t)ntasks));
    GCN_TRY(device_alloc_t(&w.task_order, (size_t)ntasks));
    TempBuf ids, len, len_sorted, plen;
    GCN_TRY(ids.alloc((size_t)ntasks * 4));
    GCN_TRY(len.alloc((size_t)ntasks * 4));
    GCN_TRY(len_sorted.alloc((size_t)ntasks * 4));
    GCN_TRY(plen.alloc((size_t)ntasks * 8));
    hipLaunchKernelGGL(k_sweep_pack, dim3(blocks_for(ntasks, 64)), dim3(64), 0, s, ntasks, rb, groups, seg.as<int64_t>(),
                       p1.as<SweepPayload>(), (const int64_t*)nullptr, (int32_t*)nullptr, (float*)nullptr,
                       (uint8_t*)nullptr, w.task_len, len.as<uint32_t>(), plen.as<int64_t>());
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_iota_i32, dim3(blocks_for(ntasks)), dim3(TPB), 0, s, ntasks, ids.as<int32_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY((prims::sort_pairs_descending<uint32_t, int32_t>(len.as<uint32_t>(), len_sorted.as<uint32_t>(),
                                                             ids.as<int32_t>(), w.task_order, (size_t)ntasks, 32u, s)));
    GCN_TRY(prims::exclusive_scan<int64_t>(plen.as<int64_t>(), w.task_base, (size_t)ntasks, s));
    int64_t nnz_light = 0, last_base = 0, last_plen = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&nnz_light, seg.as<int64_t>() + ntasks, 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipMemcpyAsync(&last_base, w.task_base + (ntasks - 1), 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipMemcpyAsync(&last_plen, plen.as<int64_t>() + (ntasks - 1), 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    const int64_t nnz_heavy = nnz - nnz_light;
    const int64_t padded = last_base + last_plen;
    w.padded = padded;

    GCN_TRY(device_alloc_t(&w.colidx, (size_t)padded));
    GCN_TRY(device_alloc_t(&w.val, (size_t)padded));
    GCN_TRY(device_alloc_t(&w.lrow, (size_t)padded));
    if (padded > 0) {
        GCN_HIP_TRY(hipMemsetAsync(w.colidx, 0xff, (size_t)padded * 4, s));  // column -1: padding until written
        GCN_HIP_TRY(hipMemsetAsync(w.val, 0, (size_t)padded * 4, s));
        GCN_HIP_TRY(hipMemsetAsync(w.lrow, 0, (size_t)padded, s));
    }
    if (nnz_light > 0) {
        // pass 2: the same walk, now writing the entries
        hipLaunchKernelGGL(k_sweep_pack, dim3(blocks_for(ntasks, 64)), dim3(64), 0, s, ntasks, rb, groups, seg.as<int64_t>(),
                           p1.as<SweepPayload>(), w.task_base, w.colidx, w.val, w.lrow, (int32_t*)nullptr,
                           (uint32_t*)nullptr, (int64_t*)nullptr);
        GCN_LAUNCH_CHECK();
    }
    if (nnz_heavy > 0) {
        Matrix* h = new (std::nothrow) Matrix();
        if (!h) return fail(GCN_ERR_OOM, "host allocation failed");
        w.heavy = h;
        GCN_TRY(device_alloc_t(&h->colidx, (size_t)nnz_heavy));
        GCN_TRY(device_alloc_t(&h->val, (size_t)nnz_heavy));
        hipLaunchKernelGGL(k_sweep_unpack, dim3(blocks_for(nnz_heavy)), dim3(TPB), 0, s, nnz_heavy, nnz_light,
                           p1.as<SweepPayload>(), h->colidx, h->val);
        GCN_LAUNCH_CHECK();
        // the heavy rows in ascending order, and their offsets into the heavy entry arrays
        TempBuf hl;
        GCN_TRY(device_alloc_t(&h->ne_rows, (size_t)(nnz_heavy / (heavy_th + 1)) + 1));
        HeavyRow pred{m.rowptr, heavy_th};
        int64_t nh_sel = 0;
        GCN_TRY(prims::select_indices(n, pred, h->ne_rows, &nh_sel, s));
        const size_t nh = (size_t)nh_sel;
        h->n_ne = nh_sel;
        GCN_TRY(hl.alloc((nh + 1) * 8));
        GCN_TRY(device_alloc_t(&h->ne_rowptr, nh + 1));
        hipLaunchKernelGGL(k_heavy_len, dim3(blocks_for((int64_t)nh + 1)), dim3(TPB), 0, s, (int64_t)nh, h->ne_rows, m.rowptr,
                           hl.as<int64_t>());
        GCN_LAUNCH_CHECK();
        GCN_TRY(prims::exclusive_scan<int64_t>(hl.as<int64_t>(), h->ne_rowptr, nh + 1, s));
        // as a compact matrix of its own: nh rows, rowptr = the offsets just computed
        h->nrows = (int64_t)nh;
        h->ncols = m.ncols;
        GCN_TRY(device_alloc_t(&h->rowptr, nh + 1));
        GCN_HIP_TRY(hipMemcpyAsync(h->rowptr, h->ne_rowptr, (nh + 1) * sizeof(int64_t), hipMemcpyDeviceToDevice, s));
        h->nsub = (nnz_heavy + SUB - 1) / SUB;
        h->nchunks = (nnz_heavy + CHUNK - 1) / CHUNK;
        const size_t padded = (size_t)h->nsub + SUBS_PER_CHUNK;
        GCN_TRY(device_alloc_t(&h->flags, padded));
        GCN_TRY(device_alloc_t(&h->sub_row, padded));
        GCN_HIP_TRY(hipMemsetAsync(h->flags, 0, padded * sizeof(uint32_t), s));
        GCN_HIP_TRY(hipMemsetAsync(h->sub_row, 0, padded * sizeof(int32_t), s));
        hipLaunchKernelGGL(k_row_flags, dim3(blocks_for(h->n_ne)), dim3(TPB), 0, s, h->n_ne, h->ne_rowptr, h->flags);
        GCN_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_sub_rows, dim3(blocks_for(h->nsub)), dim3(TPB), 0, s, h->nsub, h->n_ne, h->ne_rowptr, h->sub_row);
        GCN_LAUNCH_CHECK();
        GCN_HIP_TRY(hipStreamSynchronize(s));
        GCN_TRY(build_fix_list(h->flags, h->sub_row, h->ne_rowptr, h->nchunks, &h->fix_list, &h->n_fix, s));
    }
    GCN_HIP_TRY(hipStreamSynchronize(s));
    w.groups = groups;
    w.rb = rb;
    w.heavy_threshold = heavy_th;
    w.ntasks = ntasks;
    w.nnz_light = nnz_light;
    w.nnz_heavy = nnz_heavy;
    w.n_heavy = w.heavy ? w.heavy->n_ne : 0;
    return GCN_OK;
}

// ---- hub copy --------------------------------------------------------------------------------------------

__global__ void k_col_count(int64_t nnz, const int32_t* __restrict__ colidx, int32_t* __restrict__ cnt) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < nnz) atomicAdd(cnt + colidx[k], 1);           // integer counts: the order does not matter
}

__global__ void k_hub_rank(int64_t H, const int32_t* __restrict__ hot_col, int32_t* __restrict__ rank) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < H) rank[hot_col[r]] = (int32_t)r;
}

__global__ void k_hub_defer(int64_t n, const int64_t* __restrict__ rowptr, int32_t dmin, uint8_t* __restrict__ defer) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) defer[i] = rowptr[i + 1] - rowptr[i] >= dmin ? 1 : 0;
}

// flag[k] = 1 when entry k belongs to A_hot (long row, hot column); flag[nnz] = 0.
__global__ void k_hub_flags(int64_t nnz, int64_t n, const int64_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                            const uint8_t* __restrict__ defer, const int32_t* __restrict__ rank,
                            int64_t* __restrict__ flag) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k > nnz) return;
    if (k == nnz) { flag[k] = 0; return; }
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= k) lo = mid; else hi = mid;
    }
    flag[k] = (defer[lo] && rank[colidx[k]] >= 0) ? 1 : 0;
}

// pos = exclusive prefix sums of flag: entry k goes to A_hot[pos[k]] or to A_rest[k - pos[k]].
__global__ void k_hub_scatter(int64_t nnz, const int32_t* __restrict__ colidx, const float* __restrict__ val,
                              const int64_t* __restrict__ flag, const int64_t* __restrict__ pos,
                              const int32_t* __restrict__ rank, int32_t* __restrict__ hot_colidx,
                              float* __restrict__ hot_val, int32_t* __restrict__ rest_colidx, float* __restrict__ rest_val) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nnz) return;
    const int32_t c = colidx[k];
    if (flag[k]) {
        hot_colidx[pos[k]] = rank[c];
        hot_val[pos[k]] = val[k];
    } else {
        rest_colidx[k - pos[k]] = c;
        rest_val[k - pos[k]] = val[k];
    }
}

__global__ void k_hub_rest_rowptr(int64_t n, const int64_t* __restrict__ rowptr, const int64_t* __restrict__ pos,
                                  int64_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= n) out[i] = rowptr[i] - pos[rowptr[i]];
}

__global__ void k_hub_hot_rowptr(int64_t nh, int64_t nnz_hot, const int32_t* __restrict__ heavy_rows,
                                 const int64_t* __restrict__ rowptr, const int64_t* __restrict__ pos,
                                 int64_t* __restrict__ out) {
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nh) out[q] = pos[rowptr[heavy_rows[q]]];
    if (q == nh) out[q] = nnz_hot;
}

void free_hub(Hub& h);

int build_hub(Matrix& m, int64_t nnz, int64_t H, int64_t cpb, int32_t dmin, hipStream_t s) {
    count_build();
    free_hub(m.hub);
    Hub& h = m.hub;
    h.state = -1;                                            // until everything below has succeeded
    h.H = H; h.cpb = cpb; h.dmin = dmin;
    const int64_t n = m.nrows, nc = m.ncols;
    if (nnz <= 0 || H <= 0 || cpb <= 0 || H % cpb != 0 || H > nc || dmin < 1)
        return fail(GCN_ERR_BADARG, "build_hub: bad parameters");
    TempBuf cnt, cnt_sorted, ids, cols_sorted, rank, flag, pos, hc;

    // the H columns with the most entries, in descending order of length
    GCN_TRY(cnt.alloc((size_t)nc * 4));
    GCN_TRY(cnt_sorted.alloc((size_t)nc * 4));
    GCN_TRY(ids.alloc((size_t)nc * 4));
    GCN_TRY(cols_sorted.alloc((size_t)nc * 4));
    GCN_HIP_TRY(hipMemsetAsync(cnt.p, 0, (size_t)nc * 4, s));
    hipLaunchKernelGGL(k_col_count, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, m.colidx, cnt.as<int32_t>());
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_iota_i32, dim3(blocks_for(nc)), dim3(TPB), 0, s, nc, ids.as<int32_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY((prims::sort_pairs_descending<uint32_t, int32_t>(cnt.as<uint32_t>(), cnt_sorted.as<uint32_t>(), ids.as<int32_t>(),
                                                             cols_sorted.as<int32_t>(), (size_t)nc, 32u, s)));
    GCN_TRY(hc.alloc((size_t)H * 4));
    GCN_HIP_TRY(hipMemcpyAsync(hc.p, cols_sorted.p, (size_t)H * 4, hipMemcpyDeviceToDevice, s));
    GCN_TRY(rank.alloc((size_t)nc * 4));
    GCN_HIP_TRY(hipMemsetAsync(rank.p, 0xff, (size_t)nc * 4, s));                 // -1: not a hot column
    hipLaunchKernelGGL(k_hub_rank, dim3(blocks_for(H)), dim3(TPB), 0, s, H, hc.as<int32_t>(), rank.as<int32_t>());
    GCN_LAUNCH_CHECK();

    // the long rows
    TempBuf defer, hrows;
    GCN_TRY(defer.alloc((size_t)n));
    hipLaunchKernelGGL(k_hub_defer, dim3(blocks_for(n)), dim3(TPB), 0, s, n, m.rowptr, dmin, defer.as<uint8_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY(hrows.alloc((size_t)(nnz / dmin + 1) * 4));
    HeavyRow pred{m.rowptr, dmin - 1};
    int64_t nh_sel = 0;
    GCN_TRY(prims::select_indices(n, pred, hrows.as<int32_t>(), &nh_sel, s));
    const size_t nh = (size_t)nh_sel;
    if (nh == 0) return GCN_OK;                              // rejected: no long rows

    // split the entries
    GCN_TRY(flag.alloc(((size_t)nnz + 1) * 8));
    GCN_TRY(pos.alloc(((size_t)nnz + 1) * 8));
    hipLaunchKernelGGL(k_hub_flags, dim3(blocks_for(nnz + 1)), dim3(TPB), 0, s, nnz, n, m.rowptr, m.colidx,
                       defer.as<uint8_t>(), rank.as<int32_t>(), flag.as<int64_t>());
    GCN_LAUNCH_CHECK();
    GCN_TRY(prims::exclusive_scan<int64_t>(flag.as<int64_t>(), pos.as<int64_t>(), (size_t)nnz + 1, s));
    int64_t nnz_hot = 0;
    GCN_HIP_TRY(hipMemcpyAsync(&nnz_hot, pos.as<int64_t>() + nnz, 8, hipMemcpyDeviceToHost, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    const int64_t nnz_rest = nnz - nnz_hot;
    h.nnz_hot = nnz_hot; h.nnz_rest = nnz_rest; h.n_heavy = (int64_t)nh;
    if (nnz_hot * 2 < nnz || nnz_rest <= 0) return GCN_OK;   // rejected: less than half of the entries would gain

    Matrix* hot = new (std::nothrow) Matrix();
    Matrix* rest = new (std::nothrow) Matrix();
    h.hot = hot; h.rest = rest;
    if (!hot || !rest) return fail(GCN_ERR_OOM, "host allocation failed");
    hot->nrows = (int64_t)nh; hot->ncols = H;
    rest->nrows = n; rest->ncols = nc;
    GCN_TRY(device_alloc_t(&hot->rowptr, nh + 1));
    GCN_TRY(device_alloc_t(&hot->colidx, (size_t)nnz_hot));
    GCN_TRY(device_alloc_t(&hot->val, (size_t)nnz_hot));
    GCN_TRY(device_alloc_t(&rest->rowptr, (size_t)n + 1));
    GCN_TRY(device_alloc_t(&rest->colidx, (size_t)nnz_rest));
    GCN_TRY(device_alloc_t(&rest->val, (size_t)nnz_rest));
    hipLaunchKernelGGL(k_hub_scatter, dim3(blocks_for(nnz)), dim3(TPB), 0, s, nnz, m.colidx, m.val, flag.as<int64_t>(),
                       pos.as<int64_t>(), rank.as<int32_t>(), hot->colidx, hot->val, rest->colidx, rest->val);
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_hub_rest_rowptr, dim3(blocks_for(n + 1)), dim3(TPB), 0, s, n, m.rowptr, pos.as<int64_t>(),
                       rest->rowptr);
    GCN_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_hub_hot_rowptr, dim3(blocks_for((int64_t)nh + 1)), dim3(TPB), 0, s, (int64_t)nh, nnz_hot,
                       hrows.as<int32_t>(), m.rowptr, pos.as<int64_t>(), hot->rowptr);
    GCN_LAUNCH_CHECK();
    GCN_HIP_TRY(hipStreamSynchronize(s));
    flag.alloc(16);
    pos.alloc(16);
    GCN_TRY(build_schedule(*rest, n, nnz_rest, s));
    hot->nsub = (nnz_hot + SUB - 1) / SUB;
    hot->nchunks = (nnz_hot + CHUNK - 1) / CHUNK;
    GCN_TRY(build_blocked(*hot, nnz_hot, cpb, s));

    GCN_TRY(device_alloc_t(&h.hot_col, (size_t)H));
    GCN_TRY(device_alloc_t(&h.heavy_rows, nh));
    GCN_TRY(device_alloc_t(&h.defer, (size_t)n));
    GCN_HIP_TRY(hipMemcpyAsync(h.hot_col, hc.p, (size_t)H * 4, hipMemcpyDeviceToDevice, s));
    GCN_HIP_TRY(hipMemcpyAsync(h.heavy_rows, hrows.p, nh * 4, hipMemcpyDeviceToDevice, s));
    GCN_HIP_TRY(hipMemcpyAsync(h.defer, defer.p, (size_t)n, hipMemcpyDeviceToDevice, s));
    GCN_HIP_TRY(hipStreamSynchronize(s));
    h.state = 1;
    return GCN_OK;
}

}  // namespace gcn
